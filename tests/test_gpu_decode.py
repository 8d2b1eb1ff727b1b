"""Parity of lamps_decode_attn (through the C ABI) with the CPU oracle."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
from rig import Rig, n2t, t2n, to_f64, tol

pytestmark = pytest.mark.gpu


def _logical(seed, geom, ctx):
    K, V = [], []
    for r, c in enumerate(ctx):
        k, v = W.logical_kv(seed + 31 * (r + 1), geom, c)
        K.append(k)
        V.append(v)
    return K, V


def _setup(seed, geom, ctx, part_tokens=0):
    """Logical-first inputs paged through a seeded random block table."""
    B = len(ctx)
    rig = Rig(geom, max_batch=B, part_tokens=part_tokens)
    perm = W.permutation(seed, geom.num_blocks)
    table, _ = W.deal_block_table(perm, ctx, geom)
    K, V = _logical(seed, geom, ctx)
    q = W.queries(seed, geom, B)
    for layer in range(geom.num_layers):
        rig.page_requests(layer, table, K, V)
    return rig, table, q, K, V


CASES = [
    # dtype  H  Hkv  D   bs  part  contexts
    ("f32", 8, 8, 64, 16, 0, [17, 64, 130, 200]),
    ("f32", 8, 8, 64, 16, 32, [17, 64, 130, 200, 1, 0, 33]),
    ("f32", 4, 2, 128, 16, 64, [5, 100, 16, 129]),
    ("f32", 6, 2, 32, 32, 32, [31, 32, 33, 97]),
    ("bf16", 8, 8, 128, 16, 0, [1, 15, 16, 17, 300, 513]),
    ("bf16", 8, 2, 128, 16, 64, [2, 63, 64, 65, 200, 0]),
    ("bf16", 16, 2, 128, 32, 64, [40, 129, 7]),
    ("bf16", 4, 4, 64, 16, 32, [3, 50, 96]),
    ("bf16", 6, 3, 256, 16, 48, [20, 77]),
    ("bf16", 10, 2, 128, 16, 32, [90, 11]),
    # grouped bf16 heads (matrix-core path): group sizes 2..32, all head dims, larger blocks
    ("bf16", 8, 2, 64, 16, 32, [1, 16, 17, 100, 0]),
    ("bf16", 4, 2, 256, 16, 64, [33, 5]),
    ("bf16", 32, 1, 128, 16, 64, [70, 129]),          # 32 heads per kv head: two passes of 16
    ("bf16", 6, 2, 128, 64, 128, [63, 64, 65, 200]),
    ("bf16", 16, 1, 128, 32, 0, [31, 300]),
    ("bf16", 12, 2, 64, 16, 0, [15, 47, 2]),
    ("f32", 8, 2, 64, 16, 48, [100, 3, 49]),          # fp32 groups stay on the vector ALUs
]


# every case under both work decompositions: fixed partitions (part > 0) and balanced shares (0)
BOTH = CASES + [c[:5] + (0,) + c[6:] for c in CASES if c[5] != 0]


@pytest.mark.parametrize("dtype,H,Hkv,D,bs,part,ctx", BOTH)
def test_small_parity(dtype, H, Hkv, D, bs, part, ctx):
    mb = max(1, max((c + bs - 1) // bs for c in ctx))
    nb = sum((c + bs - 1) // bs for c in ctx) + 5
    geom = W.Geometry(2, H, Hkv, D, bs, nb, mb, dtype)
    rig, table, q, K, V = _setup(4242 + D + H, geom, ctx, part)
    B = len(ctx)
    running = np.ones(B, dtype=np.uint8)
    if B > 2:
        running[1] = 0                                   # one paused request
    for layer in (0, 1):
        out = rig.decode(layer, q, table, ctx, running, sentinel=7.0)
        ref = oracle.decode_attn(q, K, V, ctx, running)
        got = to_f64(out)
        for r in range(B):
            if running[r]:
                err = np.abs(got[r] - ref[r]).max()
                assert err <= tol(geom), (layer, r, ctx[r], err)
            else:
                assert (got[r] == 7.0).all()             # paused row untouched
    rig.close()


def test_cfg0_swap_scenario():
    """Tiny fp32 step with request 2 in Swap state: (i) swapped out, freed,
    blocks poisoned, step with it paused; (ii) swapped back into different
    blocks, all four running."""
    wl = W.workload(0)
    geom = wl.geom
    ctx = wl.ctx_lens.tolist()
    seed = W.config_seed(0)
    rig = Rig(geom, max_batch=4)
    lam = rig.lamps
    perm = W.permutation(seed, geom.num_blocks)
    # the library hands out 0,1,2,...; take all 64 and keep the first 28 of the permutation
    all_ids = lam.alloc_blocks(geom.num_blocks)
    assert all_ids == list(range(geom.num_blocks))
    table, used = W.deal_block_table(perm, ctx, geom)
    assert used == 28
    lam.free_blocks([int(b) for b in perm[used:]])
    K, V = _logical(seed, geom, ctx)
    q = W.queries(seed, geom, 4)
    rig.page_requests(0, table, K, V)

    ref = oracle.decode_attn(q, K, V, ctx, [1, 1, 1, 1])
    base = rig.decode(0, q, table, ctx, [1, 1, 1, 1])
    assert np.abs(to_f64(base) - ref).max() <= 1e-5

    # (i) request 2 enters its API call under Swap
    ids2 = [int(b) for b in table[2, :geom.blocks_for(ctx[2])]]
    host = torch.empty(len(ids2) * 2 * geom.block_half_bytes, dtype=torch.uint8).pin_memory()
    t_out = lam.swap_out(ids2, host)
    free_before = lam.num_free()
    lam.free_blocks(ids2)
    assert lam.num_free() == free_before + len(ids2)
    lam.ticket_wait(t_out)
    rig.k_pool[torch.as_tensor(ids2, device=rig.dev)] = float("nan")   # freed blocks are undefined
    rig.v_pool[torch.as_tensor(ids2, device=rig.dev)] = float("nan")
    torch.cuda.synchronize()
    out = rig.decode(0, q, table, ctx, [1, 1, 0, 1], sentinel=-5.0)
    got = to_f64(out)
    assert (got[2] == -5.0).all()
    for r in (0, 1, 3):
        assert np.abs(got[r] - ref[r]).max() <= 1e-5

    # (ii) the API returns: different physical blocks, then all four run
    pad = lam.alloc_blocks(len(ids2))                   # LIFO would return the same ids: hold them
    new_ids = lam.alloc_blocks(len(ids2))
    assert not set(new_ids) & set(ids2)
    lam.free_blocks(pad)
    t_in = lam.swap_in(host, new_ids)
    lam.compute_wait(t_in)
    table2 = table.copy()
    table2[2, :len(new_ids)] = new_ids
    out2 = rig.decode(0, q, table2, ctx, [1, 1, 1, 1])
    assert np.abs(to_f64(out2) - ref).max() <= 1e-5
    assert torch.equal(out2, base)                       # bit-identical to the pre-swap result
    rig.close()


def test_permuted_placement_is_bit_identical():
    geom = W.Geometry(1, 8, 2, 128, 16, 80, 24, "bf16")
    ctx = [333, 17, 129]
    outs = []
    for seed in (1, 2):
        rig = Rig(geom, max_batch=3, part_tokens=64)
        perm = W.permutation(seed, geom.num_blocks)
        table, _ = W.deal_block_table(perm, ctx, geom)
        K, V = _logical(77, geom, ctx)
        q = W.queries(77, geom, 3)
        rig.page_requests(0, table, K, V)
        a = rig.decode(0, q, table, ctx, [1, 1, 1])
        b = rig.decode(0, q, table, ctx, [1, 1, 1])
        assert torch.equal(a, b)                         # run-to-run reproducible
        outs.append(a.cpu())
        rig.close()
    assert torch.equal(outs[0], outs[1])


def test_unused_table_entries_and_blocks_are_never_read():
    geom = W.Geometry(1, 4, 4, 128, 16, 40, 8, "bf16")
    ctx = [50, 9]
    rig, table, q, K, V = _setup(5, geom, ctx, 32)
    ref = oracle.decode_attn(q, K, V, ctx, [1, 1])
    table = table.copy()
    table[table < 0] = 2 ** 30                           # garbage far outside the pool
    out = rig.decode(0, q, table, ctx, [1, 1])
    assert np.abs(to_f64(out) - ref).max() <= 2e-2
    rig.close()


@pytest.mark.parametrize("dtype,H,Hkv,part", [("f32", 4, 4, 0), ("bf16", 4, 4, 32), ("bf16", 8, 2, 0)])
def test_context_length_beyond_the_table_row_is_clamped(dtype, H, Hkv, part):
    """A context length larger than max_blocks_per_req * block_size is the caller's mistake; the
    kernels clamp it to the row, so no lookup leaves the block table: the result is attention
    over the row's positions."""
    geom = W.Geometry(1, H, Hkv, 64, 16, 12, 4, dtype)   # rows of 4 blocks = 64 positions
    ctx = [64, 30]
    rig, table, q, K, V = _setup(21, geom, ctx, part)
    ref = oracle.decode_attn(q, K, V, ctx, [1, 1])
    out = rig.decode(0, q, table, [64 + 5000, 30], [1, 1])
    assert np.abs(to_f64(out) - ref).max() <= tol(geom)
    rig.close()


def test_scale_override():
    geom = W.Geometry(1, 4, 4, 64, 16, 10, 4, "f32")
    ctx = [40]
    B = 1
    rig = Rig(geom, max_batch=B, scale=0.3)
    perm = W.permutation(9, geom.num_blocks)
    table, _ = W.deal_block_table(perm, ctx, geom)
    K, V = _logical(9, geom, ctx)
    q = W.queries(9, geom, B)
    rig.page_requests(0, table, K, V)
    out = rig.decode(0, q, table, ctx, [1])
    ref = oracle.decode_attn(q, K, V, ctx, [1], scale=0.3)
    assert np.abs(to_f64(out) - ref).max() <= 1e-5
    rig.close()


def _full_size(cfg, sample_requests, rep=0, part_tokens=None):
    """Physical-first: pools filled iid on the device, block table random over
    the pool; a seeded sample of running requests is un-paged for the oracle."""
    wl = W.workload(cfg, rep)
    geom = wl.geom
    seed = W.config_seed(cfg, rep)
    rig = Rig(geom, max_batch=wl.batch, poison=False,
              part_tokens=wl.part_tokens if part_tokens is None else part_tokens)
    gen = torch.Generator(device=rig.dev).manual_seed(seed)
    rig.k_pool.normal_(generator=gen)
    rig.v_pool.normal_(generator=gen)
    perm = W.permutation(seed + 3, geom.num_blocks)
    table, _ = W.deal_block_table(perm, wl.ctx_lens, geom)
    q = torch.empty((wl.batch, geom.num_q_heads, geom.head_dim), dtype=rig.tdtype,
                    device=rig.dev).normal_(generator=gen)
    running = (wl.state == W.RUNNING).astype(np.uint8)
    run_idx = np.flatnonzero(running)
    ragged, boundary = _edge_requests(wl, run_idx)
    out = rig.decode(0, q, table, wl.ctx_lens, running, sentinel=3.0)
    got = to_f64(out)
    qn = t2n(q)
    pick = run_idx[W.permutation(seed + 4, len(run_idx))[:sample_requests]]
    # always include the shortest and the longest running request, one whose length is not a
    # multiple of the kernels' chunk and one that ends exactly at a block boundary
    pick = set(pick.tolist()) | {int(run_idx[np.argmin(wl.ctx_lens[run_idx])]),
                                 int(run_idx[np.argmax(wl.ctx_lens[run_idx])]), ragged, boundary}
    worst = 0.0
    for r in sorted(pick):
        C = int(wl.ctx_lens[r])
        k, v = rig.unpage_request(0, table[r], C)
        ref = oracle.decode_attn(qn[r:r + 1], [k], [v], [C], [1], threads=8)
        worst = max(worst, np.abs(got[r] - ref[0]).max())
    paused = np.flatnonzero(running == 0)
    assert (got[paused] == 3.0).all()
    assert not np.isnan(got[run_idx]).any()
    rig.close()
    return worst


def _edge_requests(wl, run_idx):
    """A running request whose length is no multiple of 32 (the largest chunk of the kernels), and
    one whose length is a multiple of the block size -- if the draw holds none of the latter, the
    first running request is cut back to its last block boundary (in wl, before the launch)."""
    bs = wl.geom.block_size
    ragged = next(int(r) for r in run_idx if wl.ctx_lens[r] % 32 != 0)
    at = [int(r) for r in run_idx if wl.ctx_lens[r] % bs == 0 and int(r) != ragged]
    if not at:
        r = next(int(r) for r in run_idx if int(r) != ragged and wl.ctx_lens[r] >= 2 * bs)
        wl.ctx_lens[r] -= wl.ctx_lens[r] % bs
        at = [r]
    assert wl.ctx_lens[ragged] % 32 != 0 and wl.ctx_lens[at[0]] % bs == 0
    return ragged, at[0]


@pytest.mark.parametrize("cfg,sample,part", [(1, 6, None), (2, 8, None), (3, 2, None), (3, 2, 512),
                                             (1, 4, 512), (2, 6, 1024)])
def test_full_size_sampled_parity(cfg, sample, part):
    """Configurations 1-3 at full size in the bench's launch configuration
    (part=None: the workload's own setting) and in the other decomposition."""
    worst = _full_size(cfg, sample, part_tokens=part)
    assert worst <= 2e-2, worst


def test_cfg4_full_size_layers_sampled():
    """The 40-layer configuration at full size (about 110 GB of pools): layers
    0, 19 and 39, a seeded sample of running requests each."""
    wl = W.workload(4)
    geom = wl.geom
    seed = W.config_seed(4)
    free, _ = torch.cuda.mem_get_info()
    need = 2 * geom.num_blocks * geom.block_half_bytes
    if free < need * 1.05:
        pytest.skip("needs %.0f GB of free HBM" % (need / 1e9))
    rig = Rig(geom, max_batch=wl.batch, poison=False)
    gen = torch.Generator(device=rig.dev).manual_seed(seed)
    rig.k_pool.normal_(generator=gen)
    rig.v_pool.normal_(generator=gen)
    perm = W.permutation(seed + 3, geom.num_blocks)
    table, _ = W.deal_block_table(perm, wl.ctx_lens, geom)
    q = torch.empty((wl.batch, geom.num_q_heads, geom.head_dim), dtype=rig.tdtype,
                    device=rig.dev).normal_(generator=gen)
    qn = t2n(q)
    running = (wl.state == W.RUNNING).astype(np.uint8)
    run_idx = np.flatnonzero(running)
    ragged, boundary = _edge_requests(wl, run_idx)
    for layer in (0, 19, 39):
        out = rig.decode(layer, q, table, wl.ctx_lens, running, sentinel=3.0)
        got = to_f64(out)
        pick = run_idx[W.permutation(seed + 10 + layer, len(run_idx))[:6]].tolist() + [ragged, boundary]
        for r in pick:
            C = int(wl.ctx_lens[r])
            k, v = rig.unpage_request(layer, table[r], C)
            ref = oracle.decode_attn(qn[r:r + 1], [k], [v], [C], [1], threads=8)
            assert np.abs(got[r] - ref[0]).max() <= 2e-2, (layer, r)
        assert (got[running == 0] == 3.0).all()
    rig.close()


@pytest.mark.parametrize("dtype,H,Hkv", [("bf16", 4, 4), ("bf16", 8, 2), ("f32", 4, 2)])
def test_large_batch_of_short_requests(dtype, H, Hkv):
    """More requests than threads in a workgroup (the chunk-count scan then takes
    several requests per thread), most of them short, some empty, some paused."""
    B = 700
    seed = 909
    ctx = (W.splitmix64(seed, B) % np.uint64(70)).astype(np.int64)       # 0..69 tokens
    ctx[::97] = 0
    running = np.ones(B, dtype=np.uint8)
    running[::13] = 0
    geom = W.Geometry(1, H, Hkv, 64 if dtype == "f32" else 128, 16,
                      int(sum((c + 15) // 16 for c in ctx)) + 3, 5, dtype)
    rig, table, q, K, V = _setup(seed, geom, ctx.tolist())
    out = rig.decode(0, q, table, ctx, running, sentinel=2.5)
    ref = oracle.decode_attn(q, K, V, ctx, running, threads=8)
    got = to_f64(out)
    live = running == 1
    assert np.abs(got[live] - ref[live]).max() <= tol(geom)
    assert (got[~live] == 2.5).all()
    assert (got[live & (ctx == 0)] == 0).all()
    rig.close()


@pytest.mark.parametrize("dtype,H,Hkv,D,ctx", [
    ("bf16", 2, 2, 128, [40000]),                 # one request: 1 250 one-chunk pieces per head
    ("bf16", 8, 2, 128, [20000, 9000, 0]),        # matrix-core path, four heads per pass
    ("bf16", 4, 4, 64, [33000, 17]),
    ("f32", 2, 1, 64, [30000]),                   # fp32 group of two
    ("bf16", 2, 2, 128, [10000, 50]),             # longest range 313 chunks: two chunks per share
    ("bf16", 4, 4, 128, [20000, 7, 300]),         # 625 chunks: four per share
    ("bf16", 8, 2, 128, [5000, 4200]),            # matrix-core path, 313 chunks of 16 tokens
])
def test_small_batch_of_long_contexts(dtype, H, Hkv, D, ctx):
    """A few long requests: every (request, head) range is cut into hundreds of pieces,
    more than one pass of the merge's piece list, and the merge takes the pieces of a
    range in parallel."""
    seed = 1234 + H
    per = [(c + 15) // 16 for c in ctx]
    geom = W.Geometry(1, H, Hkv, D, 16, sum(per) + 5, max(per), dtype)
    rig, table, q, K, V = _setup(seed, geom, ctx)
    running = np.ones(len(ctx), dtype=np.uint8)
    out = rig.decode(0, q, table, ctx, running, sentinel=2.5)
    ref = oracle.decode_attn(q, K, V, ctx, running, threads=8)
    got = to_f64(out)
    assert np.abs(got - ref).max() <= tol(geom)
    rig.close()


@pytest.mark.parametrize("dtype,H,Hkv,D", [("bf16", 2, 2, 128), ("bf16", 8, 2, 128), ("f32", 4, 4, 64)])
def test_one_long_request_among_many_short_ones(dtype, H, Hkv, D):
    """The batch is large enough for the one-wavefront-per-share merge, and one request is so
    long that each of its ranges is cut into far more pieces than one pass of that merge's
    piece list holds."""
    seed = 4321 + H
    ctx = [20 + (i % 7) for i in range(35)] + [40000] + [33 - (i % 5) for i in range(35)]
    per = [(c + 15) // 16 for c in ctx]
    geom = W.Geometry(1, H, Hkv, D, 16, sum(per) + 5, max(per), dtype)
    rig, table, q, K, V = _setup(seed, geom, ctx)
    running = np.ones(len(ctx), dtype=np.uint8)
    running[3] = 0
    out = rig.decode(0, q, table, ctx, running, sentinel=2.5)
    ref = oracle.decode_attn(q, K, V, ctx, running, threads=8)
    got = to_f64(out)
    live = running == 1
    assert np.abs(got[live] - ref[live]).max() <= tol(geom)
    assert (got[~live] == 2.5).all()
    rig.close()


def test_validator_finds_bad_device_arguments():
    """lamps_validate_args reads the table, the lengths and the mask only.  The bad tables go to
    the validator alone, never to the attention call."""
    geom = W.Geometry(2, 8, 2, 128, 16, 40, 6, "bf16")
    ctx = [40, 96, 17, 0, 5]
    rig, table, q, K, V = _setup(77, geom, ctx)
    lam, dev = rig.lamps, rig.dev
    B = len(ctx)

    def check(tab, lens, mask):
        return lam.validate_args(B, torch.as_tensor(np.ascontiguousarray(tab, dtype=np.int32), device=dev),
                                 torch.as_tensor(np.asarray(lens, dtype=np.int32), device=dev),
                                 torch.as_tensor(np.asarray(mask, dtype=np.uint8), device=dev))
    ones = [1] * B
    assert check(table, ctx, ones) == (0, -1, 0, 0)             # unused entries are -1: never looked at
    bad = table.copy()
    bad[1, 5] = geom.num_blocks                                  # last used entry of request 1 (96 tokens = 6 blocks)
    assert check(bad, ctx, ones) == (1, 1, 2, geom.num_blocks)
    assert check(bad, ctx, [1, 0, 1, 1, 1]) == (0, -1, 0, 0)     # a paused request's table is not read
    bad[4, 0] = -7
    bad[2, 1] = 12345
    assert check(bad, ctx, ones) == (3, 1, 2, geom.num_blocks)   # three bad requests, the lowest is reported
    assert check(table, [40, 97, 17, 0, 5], ones) == (1, 1, 1, 97)     # longer than the row of 6 blocks
    assert check(table, [40, 96, -1, 0, 5], [0] * B) == (1, 2, 1, -1)  # a length is checked paused or not
    assert "request 2" in lam.last_error()
    rig.close()


def _random_case(k):
    """Seeded draw of a geometry and a batch: every supported head size, group size, block size,
    both decompositions, contexts from empty to several blocks, some requests paused."""
    u = W.uniform01(5150 + k, 64)
    dtype = "bf16" if u[0] < 0.7 else "f32"
    D = (64, 128, 256)[int(u[1] * 3)] if dtype == "bf16" else (32, 64, 128)[int(u[1] * 3)]
    Hkv = (1, 2, 3, 4)[int(u[2] * 4)]
    G = (1, 1, 2, 4, 5, 8, 16)[int(u[3] * 7)]
    bs = (16, 32, 64, 128)[int(u[4] * 4)]
    L = 1 + int(u[5] * 3)
    B = 1 + int(u[6] * 9)
    ctx = [int(u[10 + r] ** 2 * 700) for r in range(B)]                # skewed towards short, some 0
    running = [0 if u[30 + r] < 0.2 else 1 for r in range(B)]
    part = 0 if u[7] < 0.5 else bs * (1 + int(u[8] * 4))
    return dtype, Hkv * G, Hkv, D, bs, L, ctx, running, part


@pytest.mark.parametrize("k", range(24))
def test_randomized_geometries(k):
    dtype, H, Hkv, D, bs, L, ctx, running, part = _random_case(k)
    mb = max(1, max((c + bs - 1) // bs for c in ctx))
    geom = W.Geometry(L, H, Hkv, D, bs, sum((c + bs - 1) // bs for c in ctx) + 4, mb, dtype)
    rig, table, q, K, V = _setup(6000 + k, geom, ctx, part)
    layer = L - 1
    out = rig.decode(layer, q, table, ctx, running, sentinel=7.0)
    ref = oracle.decode_attn(q, K, V, ctx, running)
    got = to_f64(out)
    for r in range(len(ctx)):
        if running[r]:
            assert np.abs(got[r] - ref[r]).max() <= tol(geom), (k, r, ctx[r], geom)
            if ctx[r] == 0:
                assert (got[r] == 0).all()
        else:
            assert (got[r] == 7.0).all()
    assert rig.lamps.validate_args(len(ctx), torch.as_tensor(table, device=rig.dev),
                                   torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=rig.dev),
                                   torch.as_tensor(np.asarray(running, dtype=np.uint8), device=rig.dev))[0] == 0
    rig.close()
