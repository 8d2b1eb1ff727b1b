"""A whole decode iteration -- lamps_kv_append and lamps_decode_attn for every layer, the
context lengths advanced on the device (Section 2.2.1: the cache grows by one position per
iteration) -- captured once in a HIP graph and replayed: the calls enqueue kernels only (no
memset, no allocation, no host synchronisation), so a caller may capture them.  Every replay
is checked against the fp64 oracle over the oracle's own logical cache, with the program's
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
from rig import Rig, n2t, to_f64, tol

pytestmark = pytest.mark.gpu

#        dtype  H  Hkv D    bs  L  ctx, paused
CASES = [
    ("bf16", 8, 2, 128, 16, 2, [15, 16, 47, 3, 200], [3]),       # grouped heads: MFMA path, tiled layout
    ("bf16", 4, 4, 128, 16, 3, [31, 1, 64, 130], []),            # vector path
    ("f32", 4, 2, 64, 16, 2, [17, 40, 0], [1]),
]


@pytest.mark.parametrize("dtype,H,Hkv,D,bs,L,ctx,paused", CASES)
def test_decode_iteration_replayed_from_a_graph(dtype, H, Hkv, D, bs, L, ctx, paused):
    steps = 6                                          # one eager iteration, then five replays
    B = len(ctx)
    per_req = [(c + steps + bs - 1) // bs for c in ctx]
    geom = W.Geometry(L, H, Hkv, D, bs, sum(per_req) + 3, max(per_req), dtype)
    seed = 977 + D + H
    rig = Rig(geom, B)
    lam, dev = rig.lamps, rig.dev
    perm = W.permutation(seed, geom.num_blocks)
    table, _ = W.deal_block_table(perm, [c + steps for c in ctx], geom)
    K = [[W.logical_kv(seed + 100 * l + r, geom, c)[0] for r, c in enumerate(ctx)] for l in range(L)]
    V = [[W.logical_kv(seed + 100 * l + r, geom, c)[1] for r, c in enumerate(ctx)] for l in range(L)]
    for l in range(L):
        rig.page_requests(l, table, K[l], V[l])
    model = oracle.LogicalCache(L, ctx, K, V)
    running = np.ones(B, dtype=np.uint8)
    running[paused] = 0

    # everything the captured iteration touches lives in tensors allocated once
    td = torch.as_tensor(table, device=dev)
    cd = torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=dev)
    cd1 = torch.zeros_like(cd)                         # lengths including the token being generated
    md = torch.as_tensor(running, device=dev)
    q_s = torch.zeros((L, B, H, D), dtype=rig.tdtype, device=dev)
    k_s = torch.zeros((L, B, Hkv, D), dtype=rig.tdtype, device=dev)
    v_s = torch.zeros_like(k_s)
    out_s = torch.zeros_like(q_s)

    def iteration():
        torch.add(cd, 1, out=cd1)
        for l in range(L):
            lam.kv_append(l, B, k_s[l], v_s[l], td, cd, md, l == L - 1)
            lam.decode_attn(l, B, q_s[l], td, cd1, md, out_s[l])

    def inputs(it):
        qs = [W.queries(seed + 13 * it + l, geom, B) for l in range(L)]
        kv = [W.logical_kv(seed + 7919 * it + 31 * l, geom, B) for l in range(L)]
        return qs, [x[0] for x in kv], [x[1] for x in kv]

    graph = None
    for it in range(steps):
        qs, kn, vn = inputs(it)
        with torch.cuda.stream(rig.compute):           # the program's own eager work between replays
            for l in range(L):
                q_s[l].copy_(n2t(qs[l], dev))
                k_s[l].copy_(n2t(kn[l], dev))
                v_s[l].copy_(n2t(vn[l], dev))
            out_s.fill_(2.5)
            if it == 0:
                iteration()                            # eager once: nothing initialises lazily under capture
        rig.compute.synchronize()
        if it == 1:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=rig.compute):
                iteration()                            # capture enqueues nothing
        if it >= 1:
            with torch.cuda.stream(rig.compute):
                graph.replay()
        rig.compute.synchronize()
        torch.cuda.synchronize()
        got = to_f64(out_s)
        for l in range(L):
            model.append(l, kn[l], vn[l], running, l == L - 1)
        for l in range(L):
            ref = oracle.decode_attn(qs[l], model.K[l], model.V[l], model.ctx, running)
            live = running == 1
            assert np.abs(got[l][live] - ref[live]).max() <= tol(geom), (it, l)
            assert (got[l][~live] == 2.5).all(), (it, l)
        assert cd.cpu().tolist() == model.ctx, it
    rig.close()


@pytest.mark.parametrize("cfg", [1, 2])
def test_full_size_step_replayed_from_a_graph(cfg):
    """The launch configuration the benchmark times for its 40-layer headline -- every layer's
    decode call of a step replayed from one HIP graph -- at full size: configuration 1 (vector
    path) and 2 (grouped heads) with the layer call captured four times over four query / output
    buffers.  Each replay is bit-identical to the eager calls, and a seeded sample of requests is
    checked against the oracle."""
    wl = W.workload(cfg)
    geom, seed = wl.geom, W.config_seed(cfg)
    rig = Rig(geom, max_batch=wl.batch, poison=False)
    lam, dev = rig.lamps, rig.dev
    gen = torch.Generator(device=dev).manual_seed(seed)
    rig.k_pool.normal_(generator=gen)
    rig.v_pool.normal_(generator=gen)
    perm = W.permutation(seed + 3, geom.num_blocks)
    table, _ = W.deal_block_table(perm, wl.ctx_lens, geom)
    running = (wl.state == W.RUNNING).astype(np.uint8)
    td = torch.as_tensor(table, device=dev)
    cd = torch.as_tensor(wl.ctx_lens.astype(np.int32), device=dev)
    md = torch.as_tensor(running, device=dev)
    n = 4
    qs = [torch.empty((wl.batch, geom.num_q_heads, geom.head_dim), dtype=rig.tdtype, device=dev).normal_(generator=gen)
          for _ in range(n)]
    eager = [torch.full_like(q, 3.0) for q in qs]
    outs = [torch.full_like(q, 3.0) for q in qs]
    with torch.cuda.stream(rig.compute):
        for i in range(n):
            lam.decode_attn(0, wl.batch, qs[i], td, cd, md, eager[i])
    rig.compute.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=rig.compute):
        for i in range(n):
            lam.decode_attn(0, wl.batch, qs[i], td, cd, md, outs[i])
    for rep in range(3):
        for o in outs:
            o.fill_(3.0)
        torch.cuda.synchronize()                        # the program's own work and waits between replays
        with torch.cuda.stream(rig.compute):
            graph.replay()
        rig.compute.synchronize()
        for i in range(n):
            assert torch.equal(outs[i].view(torch.int16), eager[i].view(torch.int16)), (rep, i)
    run_idx = np.flatnonzero(running)
    pick = run_idx[W.permutation(seed + 21, len(run_idx))[:4]]
    got = to_f64(outs[n - 1])
    qn = qs[n - 1].cpu().view(torch.int16).numpy().view(np.uint16)
    for r in pick:
        C = int(wl.ctx_lens[r])
        k, v = rig.unpage_request(0, table[r], C)
        ref = oracle.decode_attn(qn[r:r + 1], [k], [v], [C], [1], threads=8)
        assert np.abs(got[r] - ref[0]).max() <= tol(geom), r
    assert (got[running == 0] == 3.0).all()
    rig.close()
