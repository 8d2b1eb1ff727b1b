"""lamps_decode_attn_static -- the decode call for callers that cannot allocate -- against
lamps_decode_attn on the same inputs, through the C ABI.

Both run the same kernels with the same share count, so the results are compared bit for bit
(and the existing call is itself checked against the fp64 oracle here, at the usual tolerance).
Two calls in a row share the library's static scratch array; the second is smaller, so it runs
over the first one's leftovers."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
import paper_2410_18248_amd as P
from rig import Rig, n2t, to_f64, tol

pytestmark = pytest.mark.gpu


def _case(rig, geom, seed, ctx, running):
    """Pages fresh logical K/V for `ctx` into rig's pools; returns device arguments and the oracle's result."""
    B = len(ctx)
    perm = W.permutation(seed, geom.num_blocks)
    table, _ = W.deal_block_table(perm, ctx, geom)
    K, V = [], []
    for r, c in enumerate(ctx):
        k, v = W.logical_kv(seed + 31 * (r + 1), geom, c)
        K.append(k)
        V.append(v)
    q = W.queries(seed, geom, B)
    for layer in range(geom.num_layers):
        rig.page_requests(layer, table, K, V)
    dev = rig.dev
    args = (n2t(q, dev), torch.as_tensor(np.ascontiguousarray(table, dtype=np.int32), device=dev),
            torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=dev),
            torch.as_tensor(np.asarray(running, dtype=np.uint8), device=dev))
    return args, oracle.decode_attn(q, K, V, ctx, running)


@pytest.mark.parametrize("dtype,H,Hkv,D,bs", [("bf16", 8, 8, 128, 16), ("bf16", 16, 4, 128, 16),
                                              ("f32", 8, 8, 64, 16)])
def test_static_scratch_decode_equals_the_workspace_decode_twice_in_a_row(dtype, H, Hkv, D, bs):
    big = [700, 1, 16, 2500, 333, 0, 64, 1290, 47, 900, 2048, 5]     # split ranges: long contexts, few requests
    small = [130, 9, 1100]
    mb = max((c + bs - 1) // bs for c in big)
    nb = sum((c + bs - 1) // bs for c in big) + 7
    geom = W.Geometry(2, H, Hkv, D, bs, nb, mb, dtype)
    rig = Rig(geom, max_batch=len(big))
    for ctx, seed in ((big, 9100 + D), (small, 9200 + H)):
        B = len(ctx)
        running = np.ones(B, dtype=np.uint8)
        running[1] = 0                                                # one paused request
        (q, table, lens, mask), ref = _case(rig, geom, seed, ctx, running)
        for layer in (0, 1):
            want = torch.full((B, H, D), 7.0, dtype=rig.tdtype, device=rig.dev)
            got = torch.full((B, H, D), 7.0, dtype=rig.tdtype, device=rig.dev)
            with torch.cuda.stream(rig.compute):
                rig.lamps.decode_attn(layer, B, q, table, lens, mask, want)
                P.lamps_decode_attn_static(rig.cfg, rig.compute.cuda_stream, layer, B, q, rig.k_pool,
                                           rig.v_pool, table, lens, mask, got)
            rig.compute.synchronize()
            if layer == 0:                                            # the existing call against the oracle
                w = to_f64(want)
                for r in range(B):
                    if running[r]:
                        assert np.abs(w[r] - ref[r]).max() <= tol(geom), (ctx[r],)
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), (ctx, layer)
            assert (to_f64(got)[1] == 7.0).all()                      # paused row untouched
    rig.close()


def test_static_scratch_decode_captured_in_a_graph():
    """The callers the entry point is for: one eager call first (it looks the scratch array up),
    then the call is captured into a HIP graph -- nothing in it allocates or synchronises -- and
    replayed with other work in between; every replay equals lamps_decode_attn bit for bit."""
    ctx = [900, 30, 1500, 77, 2100, 260]
    H, Hkv, D, bs = 16, 4, 128, 16
    mb = max((c + bs - 1) // bs for c in ctx)
    geom = W.Geometry(1, H, Hkv, D, bs, sum((c + bs - 1) // bs for c in ctx) + 3, mb, "bf16")
    rig = Rig(geom, max_batch=len(ctx))
    B = len(ctx)
    running = np.ones(B, dtype=np.uint8)
    (q, table, lens, mask), ref = _case(rig, geom, 9300, ctx, running)
    want = torch.zeros((B, H, D), dtype=rig.tdtype, device=rig.dev)
    got = torch.zeros_like(want)
    with torch.cuda.stream(rig.compute):
        rig.lamps.decode_attn(0, B, q, table, lens, mask, want)
        P.lamps_decode_attn_static(rig.cfg, rig.compute.cuda_stream, 0, B, q, rig.k_pool, rig.v_pool, table, lens,
                                   mask, got)                          # eager once
    rig.compute.synchronize()
    assert np.abs(to_f64(want) - ref).max() <= tol(geom)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=rig.compute):
        P.lamps_decode_attn_static(rig.cfg, rig.compute.cuda_stream, 0, B, q, rig.k_pool, rig.v_pool, table, lens,
                                   mask, got)
    for rep in range(3):
        got.fill_(5.0)
        torch.cuda.synchronize()
        with torch.cuda.stream(rig.compute):
            graph.replay()
        rig.compute.synchronize()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), rep
    rig.close()


def test_static_scratch_decode_refuses_what_it_cannot_hold():
    geom = W.Geometry(1, 64, 4, 128, 16, 8, 4, "bf16")                # 16 heads per pass: 34 MB of partial slots
    rig = Rig(geom, max_batch=2)
    z = torch.zeros(2 * 64 * 128, dtype=torch.bfloat16, device=rig.dev)
    table = torch.zeros((2, 4), dtype=torch.int32, device=rig.dev)
    lens = torch.zeros(2, dtype=torch.int32, device=rig.dev)
    mask = torch.zeros(2, dtype=torch.uint8, device=rig.dev)           # nobody runs, whatever happens
    with pytest.raises(P.LampsError) as e:
        P.lamps_decode_attn_static(rig.cfg, rig.compute.cuda_stream, 0, 2, z, rig.k_pool, rig.v_pool, table,
                                   lens, mask, z)
    assert e.value.status == -2 and "static scratch" in str(e.value)
    with pytest.raises(P.LampsError) as e:                            # batch beyond cfg.max_batch
        P.lamps_decode_attn_static(rig.cfg, rig.compute.cuda_stream, 0, 3, z, rig.k_pool, rig.v_pool, table,
                                   lens, mask, z)
    assert e.value.status == -2
    rig.close()
