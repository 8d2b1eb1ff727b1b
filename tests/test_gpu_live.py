"""The whole library under the scheduler's control: a small trace is served for real
(append, decode, swap out / in, discard + recompute, prefill of prompts and API responses)
and the attention output of EVERY processed token is compared with the fp64 oracle over the
request's logical keys and values; at the end every block is free again."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
import paper_2410_18248_amd as P
from paper_2410_18248_amd.engine import LiveEngine, RandomSource

pytestmark = pytest.mark.gpu


def _bits(t):
    t = t.contiguous()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()


@pytest.mark.parametrize("dtype,H,Hkv,policy,layered", [
    ("bf16", 4, 4, P.LAMPS_POLICY_LAMPS, False), ("bf16", 8, 2, P.LAMPS_POLICY_FCFS, False),
    ("f32", 4, 2, P.LAMPS_POLICY_SJF, False), ("bf16", 8, 2, P.LAMPS_POLICY_LAMPS, True)])
def test_trace_served_on_the_gpu_matches_the_oracle_token_by_token(dtype, H, Hkv, policy, layered):
    L, D, bs = 2, 64, 16
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    memory_tokens, n_req = 400, 10
    nb = memory_tokens // bs + n_req + 2
    cfg = P.LampsConfig(L, H, Hkv, D, bs, nb, 16, 8, P.LAMPS_BF16 if dtype == "bf16" else P.LAMPS_F32, 0.0, 0, 0)
    cost = P.LampsCostModel(1e-3, 1e-7, 1e-4, 1e-5, 1e-4, 1e-6, 0, 0)
    scfg = P.LampsSchedConfig(policy, 4, memory_tokens, 20, 1, 1 << 20, 50.0, 1.0, cost)
    src = RandomSource(77, H, Hkv, D, tdt)
    worst = [0.0]
    seen = {}

    def observer(kind, rid, layer, first_pos, rows):
        # logical keys / values of the request up to the last processed position, from the source
        n = rows.shape[0]
        q, k, v = src.rows(rid, 0, first_pos + n, layer)
        qb, kb, vb = _bits(q[first_pos:]), _bits(k), _bits(v)
        ref = oracle.decode_attn(qb, [kb] * n, [vb] * n, [first_pos + i + 1 for i in range(n)], [1] * n)
        worst[0] = max(worst[0], float(np.abs(rows.double().numpy() - ref).max()))
        seen[(rid, layer)] = seen.get((rid, layer), 0) + n

    eng = LiveEngine(cfg, scfg, src, observer=observer, layered_swap=layered)
    u = W.uniform01(5, 10 * n_req)
    want_tokens = {}
    strategies = [P.LAMPS_PRESERVE, P.LAMPS_DISCARD, P.LAMPS_SWAP]
    for i in range(n_req):
        x = u[10 * i:10 * i + 10]
        segs, toks = [], int(x[0] * 30)                 # prompt
        prompt = toks
        for k in range(1 + int(x[1] * 2)):              # one or two API calls, every strategy is used
            n_out, rho = 1 + int(x[2 + k] * 12), int(x[4 + k] * 8)
            segs.append((n_out, 0.002 + 0.01 * x[6 + k], rho, strategies[(i + k) % 3]))
            toks += n_out + rho
        n_last = 1 + int(x[8] * 10)
        segs.append((n_last, None, 0, None))
        want_tokens[i] = toks + n_last
        eng.add(i, 0.001 * i, prompt, segs)
    stats = eng.run(max_iterations=5000)
    assert eng.lam.num_free() == nb                     # every block came back
    for i in range(n_req):
        c, f, h = eng.sched.result(i, 3)
        assert c > 0 and f > 0
    # every position of every request went through attention at least once in every layer
    # (more than once where a discarded context was recomputed)
    for i in range(n_req):
        for layer in range(L):
            assert seen[(i, layer)] >= want_tokens[i], (i, layer)
    assert stats["swapped_out_blocks"] > 0 and stats["swapped_in_blocks"] > 0 and stats["discarded_blocks"] > 0
    assert worst[0] <= (1e-5 if dtype == "f32" else 2e-2), worst[0]
    eng.close()


def test_device_source_is_a_pure_function_and_serves_a_trace():
    """The device-side input source of serve_live: rows depend on (seed, rid, position, layer)
    only, whatever range they are asked for in; a short trace served with it ends with every
    block free."""
    from paper_2410_18248_amd.engine import DeviceSource
    H, Hkv, D, L, bs = 4, 2, 64, 2, 16
    src = DeviceSource(5, H, Hkv, D, torch.bfloat16)
    q, k, v = src.rows(3, 0, 9, 1)
    q2, k2, v2 = src.rows(3, 4, 5, 1)
    assert torch.equal(q[4:], q2) and torch.equal(k[4:], k2) and torch.equal(v[4:], v2)
    assert not torch.equal(src.rows(3, 0, 9, 0)[0], q) and not torch.equal(src.rows(4, 0, 9, 1)[0], q)
    big = torch.cat([x.float().flatten() for x in src.rows(1, 0, 64, 0)])
    assert abs(float(big.mean())) < 0.05 and abs(float(big.var()) - 1.0) < 0.05
    memory_tokens, n_req = 300, 6
    nb = memory_tokens // bs + n_req + 2
    cfg = P.LampsConfig(L, H, Hkv, D, bs, nb, 16, 4, P.LAMPS_BF16, 0.0, 0, 0)
    cost = P.LampsCostModel(1e-3, 1e-7, 1e-4, 1e-5, 1e-4, 1e-6, 0, 0)
    scfg = P.LampsSchedConfig(P.LAMPS_POLICY_LAMPS, 4, memory_tokens, 20, 1, 1 << 20, 50.0, 1.0, cost)
    eng = LiveEngine(cfg, scfg, src)
    for i in range(n_req):
        eng.add(i, 0.001 * i, 10 + 3 * i, [(5 + i, 0.003, 4, [P.LAMPS_PRESERVE, P.LAMPS_DISCARD, P.LAMPS_SWAP][i % 3]),
                                            (6, None, 0, None)])
    stats = eng.run(max_iterations=2000)
    assert eng.lam.num_free() == nb
    assert stats["decode_tokens"] == sum(5 + i + 6 for i in range(n_req))
    eng.close()
