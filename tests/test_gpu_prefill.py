"""GPU parity for lamps_kv_append_tokens and lamps_prefill_attn (Discard's recompute,
prompts, API responses: several new tokens per request, each attending to the cached
positions up to its own): appended pools bit-exact against the harness' pager, attention
against the fp64 oracle."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
import paper_2410_18248_amd as P
from rig import Rig, n2t, to_f64, tol

pytestmark = pytest.mark.gpu

#        dtype  H  Hkv D    bs  (context, new tokens) per request
CASES = [
    ("f32", 4, 4, 64, 16, [(40, 40), (17, 3), (64, 1), (9, 0), (33, 33)]),
    ("f32", 8, 2, 32, 16, [(50, 50), (20, 7)]),
    ("bf16", 4, 4, 128, 16, [(130, 130), (47, 5), (16, 16), (1, 1)]),
    ("bf16", 8, 2, 128, 16, [(130, 130), (47, 5), (16, 16), (1, 1), (200, 64)]),     # tiled layout
    ("bf16", 8, 2, 64, 32, [(95, 95), (64, 33)]),
    ("bf16", 16, 1, 256, 16, [(70, 70), (31, 2)]),
    ("bf16", 32, 1, 128, 16, [(45, 45), (20, 3)]),                                   # 32 heads per kv head
    ("bf16", 2, 2, 64, 64, [(150, 150)]),
    ("bf16", 4, 4, 128, 16, [(700, 700), (300, 37)]),                                # several q tiles and stages
    ("bf16", 8, 2, 128, 16, [(333, 333), (500, 100)]),
    ("bf16", 6, 2, 128, 16, [(100, 100), (77, 10)]),                                 # group of 3
    ("bf16", 4, 4, 256, 16, [(90, 90), (50, 6)]),
    # (request, kv head) pairs that do not fill groups of 8: their tiles are dealt over all XCDs
    ("bf16", 8, 1, 128, 16, [(300, 300)]),
    ("bf16", 4, 1, 64, 16, [(100, 100), (50, 50), (70, 70)]),
    ("bf16", 8, 4, 128, 16, [(100, 100), (60, 60), (40, 17)]),       # 12 pairs: a whole group of 8 and 4 left over
    ("bf16", 5, 5, 64, 16, [(150, 150)]),                            # 5 pairs
    # few new tokens per request: the waves of a workgroup split the cached positions (4 and 2 ways)
    ("bf16", 4, 4, 128, 16, [(300, 20), (150, 32), (64, 1), (33, 0)]),
    ("bf16", 4, 4, 128, 16, [(300, 50), (100, 64), (70, 3)]),
    ("bf16", 8, 2, 128, 16, [(500, 8), (100, 3), (8, 8)]),
    ("bf16", 8, 2, 64, 32, [(200, 16), (90, 9)]),
]


def _setup(dtype, H, Hkv, D, bs, reqs, seed):
    ctx = [c for c, _ in reqs]
    new = [n for _, n in reqs]
    nb = sum((c + bs - 1) // bs for c in ctx)
    geom = W.Geometry(1, H, Hkv, D, bs, nb + 4, max((c + bs - 1) // bs for c in ctx), dtype)
    rig = Rig(geom, len(reqs))
    perm = W.permutation(seed, geom.num_blocks)
    table, _ = W.deal_block_table(perm, ctx, geom)
    K, V = zip(*[W.logical_kv(seed + 17 * r, geom, c) for r, c in enumerate(ctx)])
    # what was cached before: everything but the new tokens
    rig.page_requests(0, table, [K[r][:c - n] for r, (c, n) in enumerate(reqs)],
                      [V[r][:c - n] for r, (c, n) in enumerate(reqs)])
    q_start = np.concatenate([[0], np.cumsum(new)]).astype(np.int32)
    return geom, rig, table, K, V, ctx, new, q_start


@pytest.mark.parametrize("rows_kernel", [False, True])
@pytest.mark.parametrize("dtype,H,Hkv,D,bs,reqs", CASES)
def test_append_tokens_then_prefill_attention(dtype, H, Hkv, D, bs, reqs, rows_kernel):
    """Both kernels: matrix cores where the geometry allows (bf16), and one wavefront per token."""
    seed = 9000 + D + bs + H
    geom, rig, table, K, V, ctx, new, q_start = _setup(dtype, H, Hkv, D, bs, reqs, seed)
    total = int(q_start[-1])
    dev = rig.dev
    k_new = np.concatenate([K[r][c - n:] for r, (c, n) in enumerate(reqs)])
    v_new = np.concatenate([V[r][c - n:] for r, (c, n) in enumerate(reqs)])
    q = W.queries(seed + 5, geom, total)
    td = torch.as_tensor(table, device=dev)
    cd = torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=dev)
    sd = torch.as_tensor(q_start, device=dev)
    out = torch.full((total, H, D), 7.0, dtype=rig.tdtype, device=dev)
    with torch.cuda.stream(rig.compute):
        kd, vd, qd = n2t(k_new, dev), n2t(v_new, dev), n2t(q, dev)
        rig.lamps.kv_append_tokens(0, len(reqs), total, kd, vd, sd, td, cd)
        rig.lamps.prefill_attn(0, len(reqs), total, qd, sd, td, cd, out,
                               max_new_tokens=-1 if rows_kernel else max(new))
    rig.compute.synchronize()
    # the cache now holds the full sequences, and nothing else changed
    kp = np.full(geom.pool_shape, W.poison(geom), dtype=geom.np_dtype)
    vp = kp.copy()
    for r in range(len(reqs)):
        W.page(kp, 0, table[r], K[r], rig.k_index)
        W.page(vp, 0, table[r], V[r], rig.v_index)
    got_k, got_v = rig.host_pools()
    assert got_k.tobytes() == kp.tobytes() and got_v.tobytes() == vp.tobytes()
    ref = oracle.prefill_attn(q, K, V, q_start, ctx, threads=8)
    got = to_f64(out)
    assert np.abs(got - ref).max() <= tol(geom)
    # a single new token is a decode step (another summation order: not the same bits)
    for r, (c, n) in enumerate(reqs):
        if n == 1:
            one = rig.decode(0, q[q_start[r]:q_start[r] + 1], table[r:r + 1], [c], [1])
            assert np.abs(to_f64(one)[0] - got[q_start[r]]).max() <= (1e-5 if dtype == "f32" else 2e-2)
    rig.close()


def test_prefill_is_independent_of_block_placement():
    reqs = [(77, 77), (40, 9)]
    outs = []
    for seed in (1, 2):                                 # two different random placements
        geom, rig, table, K, V, ctx, new, q_start = _setup("bf16", 8, 2, 128, 16, reqs, 500)
        perm = W.permutation(seed, geom.num_blocks)
        table, _ = W.deal_block_table(perm, ctx, geom)
        rig.k_pool.fill_(float("nan"))
        rig.v_pool.fill_(float("nan"))
        rig.page_requests(0, table, K, V)
        total = int(q_start[-1])
        q = W.queries(77, geom, total)
        dev = rig.dev
        out = torch.zeros((total, 8, 128), dtype=rig.tdtype, device=dev)
        with torch.cuda.stream(rig.compute):
            rig.lamps.prefill_attn(0, 2, total, n2t(q, dev), torch.as_tensor(q_start, device=dev),
                                   torch.as_tensor(table, device=dev),
                                   torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=dev), out)
        rig.compute.synchronize()
        outs.append(out.clone())
        rig.close()
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("rows_kernel", [False, True])
def test_prefill_leaves_impossible_contexts_alone(rows_kernel):
    """A context shorter than its new tokens, or longer than the block-table row, cannot be
    addressed: both kernels write nothing for such a request and serve the others."""
    reqs = [(40, 10), (64, 64), (33, 33)]
    geom, rig, table, K, V, ctx, new, q_start = _setup("bf16", 4, 4, 64, 16, reqs, 321)
    rig.page_requests(0, table, K, V)
    total = int(q_start[-1])
    q = W.queries(9, geom, total)
    dev = rig.dev
    bad = np.asarray([5, 64 + 7000, 33], dtype=np.int32)       # shorter than its 10 new tokens; past its 4-block row
    out = torch.full((total, 4, 64), 3.0, dtype=rig.tdtype, device=dev)
    with torch.cuda.stream(rig.compute):
        rig.lamps.prefill_attn(0, 3, total, n2t(q, dev), torch.as_tensor(q_start, device=dev),
                               torch.as_tensor(table, device=dev), torch.as_tensor(bad, device=dev), out,
                               max_new_tokens=-1 if rows_kernel else 64)
    rig.compute.synchronize()
    got = to_f64(out)
    assert (got[:74] == 3.0).all()                      # requests 0 and 1: untouched
    ref = oracle.prefill_attn(q, K, V, q_start, ctx)
    assert np.abs(got[74:] - ref[74:]).max() <= 2e-2
    rig.close()


def test_prefill_rejects_bad_host_arguments():
    geom = W.Geometry(2, 4, 4, 64, 16, 8, 2, "f32")
    rig = Rig(geom, 2)
    x = torch.zeros(8, device=rig.dev)
    for call in (rig.lamps.prefill_attn, ):
        with pytest.raises(P.LampsError) as e:
            call(2, 1, 1, x, x, x, x, x)
        assert e.value.status == -2
        with pytest.raises(P.LampsError) as e:
            call(0, 3, 1, x, x, x, x, x)
        assert e.value.status == -2
        with pytest.raises(P.LampsError) as e:
            call(0, 1, 1, None, x, x, x, x)
        assert e.value.status == -1
    with pytest.raises(P.LampsError) as e:
        rig.lamps.kv_append_tokens(0, 1, -1, x, x, x, x, x)
    assert e.value.status == -2
    rig.close()


@pytest.mark.parametrize("H,Hkv,n_req,n_new,cached", [(40, 40, 2, 4096, 0), (32, 8, 2, 4096, 0), (32, 8, 4, 512, 4096),
                                                      (32, 32, 8, 32, 1024)])
def test_full_size_sampled_prefill(H, Hkv, n_req, n_new, cached):
    """The sizes `bench.py --prefill` times (many tiles per request, hundreds of stages, the
    launch order over the XCDs): append + attention on device-generated data, sampled rows of
    the first and the last request against the oracle on the un-paged cache."""
    D, bs = 128, 16
    C = cached + n_new
    per = (C + bs - 1) // bs
    nb = n_req * per + 8
    geom = W.Geometry(1, H, Hkv, D, bs, nb, per, "bf16")
    rig = Rig(geom, n_req, poison=False)
    dev = rig.dev
    gen = torch.Generator(device=dev).manual_seed(W.config_seed(6) + H + n_new)
    rig.k_pool.normal_(generator=gen)
    rig.v_pool.normal_(generator=gen)
    perm = W.permutation(W.config_seed(6) + 1, nb)
    table, _ = W.deal_block_table(perm, [C] * n_req, geom)
    td = torch.as_tensor(table, device=dev)
    cd = torch.full((n_req,), C, dtype=torch.int32, device=dev)
    sd = torch.arange(0, (n_req + 1) * n_new, n_new, dtype=torch.int32, device=dev)
    total = n_req * n_new
    q = torch.empty((total, H, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    kn = torch.empty((total, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    vn = torch.empty((total, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    out = torch.full_like(q, 7.0)
    torch.cuda.synchronize()
    with torch.cuda.stream(rig.compute):
        rig.lamps.kv_append_tokens(0, n_req, total, kn, vn, sd, td, cd)
        rig.lamps.prefill_attn(0, n_req, total, q, sd, td, cd, out, max_new_tokens=n_new)
    rig.compute.synchronize()
    k_index, v_index = geom.tile_index_maps()
    rows = sorted(set([0, 1, 31, 32, n_new // 3, n_new // 2 + 17, n_new - 2, n_new - 1]) & set(range(n_new)))
    for r in (0, n_req - 1):
        ids = torch.as_tensor(table[r, :per].astype(np.int64), device=dev)
        K = W.tiles_to_logical(rig.k_pool[ids, 0].cpu().view(torch.int16).numpy().view(np.uint16), k_index, C)
        V = W.tiles_to_logical(rig.v_pool[ids, 0].cpu().view(torch.int16).numpy().view(np.uint16), v_index, C)
        # the appended rows are where the new keys and values were asked to go
        np.testing.assert_array_equal(K[cached:], kn[r * n_new:(r + 1) * n_new].cpu().view(torch.int16).numpy().view(np.uint16))
        np.testing.assert_array_equal(V[cached:], vn[r * n_new:(r + 1) * n_new].cpu().view(torch.int16).numpy().view(np.uint16))
        qh = q[r * n_new:(r + 1) * n_new].cpu().view(torch.int16).numpy().view(np.uint16)
        ref = oracle.decode_attn(qh[rows], [K] * len(rows), [V] * len(rows), [cached + i + 1 for i in rows], [1] * len(rows))
        got = to_f64(out[r * n_new:(r + 1) * n_new])[rows]
        np.testing.assert_allclose(got, ref, rtol=0, atol=tol(geom))
    rig.close()
