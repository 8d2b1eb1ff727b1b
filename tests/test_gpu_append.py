"""GPU parity for lamps_kv_append (the cache grows by one position per layer per
iteration, Section 2.2.1): bit-exact against the oracle's logical cache through
the harness' un-pager, no stray writes anywhere in the pools, and attention over
the grown cache against the fp64 oracle."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
from rig import Rig, n2t, t2n, to_f64, tol

pytestmark = pytest.mark.gpu

#        dtype  H  Hkv D    bs  L  ctx (some on a block boundary, one empty), paused
CASES = [
    ("f32", 4, 4, 64, 16, 1, [17, 16, 0, 31, 40], [3]),
    ("bf16", 4, 4, 128, 16, 2, [15, 16, 33, 1], [0]),
    ("bf16", 8, 2, 128, 16, 2, [15, 16, 47, 0, 20], [4]),          # tiled layout
    ("bf16", 8, 2, 64, 32, 1, [31, 32, 63, 5], []),
    ("bf16", 16, 2, 256, 16, 1, [7, 48], [1]),
    ("f32", 8, 2, 32, 64, 3, [63, 64, 100], []),
]


def _new_rows(seed, geom, B):
    k, v = W.logical_kv(seed, geom, B)                 # [B][Hkv][D] in the storage type
    return k, v


@pytest.mark.parametrize("dtype,H,Hkv,D,bs,L,ctx,paused", CASES)
def test_append_steps_match_logical_cache(dtype, H, Hkv, D, bs, L, ctx, paused):
    steps = bs + 3                                     # every request crosses a block boundary
    B = len(ctx)
    per_req = [(c + steps + bs - 1) // bs for c in ctx]
    geom = W.Geometry(L, H, Hkv, D, bs, sum(per_req) + 5, max(per_req), dtype)
    seed = 4242 + D + bs
    rig = Rig(geom, B)
    perm = W.permutation(seed, geom.num_blocks)
    # the table holds every block a request will grow into (allocation is the caller's)
    table, used = W.deal_block_table(perm, [c + steps for c in ctx], geom)
    K = [[W.logical_kv(seed + 100 * l + r, geom, c)[0] for r, c in enumerate(ctx)] for l in range(L)]
    V = [[W.logical_kv(seed + 100 * l + r, geom, c)[1] for r, c in enumerate(ctx)] for l in range(L)]
    for l in range(L):
        rig.page_requests(l, table, K[l], V[l])
    model = oracle.LogicalCache(L, ctx, K, V)
    running = np.ones(B, dtype=np.uint8)
    running[paused] = 0
    dev = rig.dev
    td = torch.as_tensor(table, device=dev)
    cd = torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=dev)
    md = torch.as_tensor(running, device=dev)
    for it in range(steps):
        for l in range(L):
            kn, vn = _new_rows(seed + 7919 * it + 31 * l, geom, B)
            with torch.cuda.stream(rig.compute):
                rig.lamps.kv_append(l, B, n2t(kn, dev), n2t(vn, dev), td, cd, md, l == L - 1)
            rig.compute.synchronize()
            model.append(l, kn, vn, running, l == L - 1)
    assert cd.cpu().tolist() == model.ctx
    # expected pools: the model's sequences paged (by the harness) over the NaN-filled pools
    kp = np.full(geom.pool_shape, W.poison(geom), dtype=geom.np_dtype)
    vp = kp.copy()
    for l in range(L):
        for r in range(B):
            W.page(kp, l, table[r], model.K[l][r], rig.k_index)
            W.page(vp, l, table[r], model.V[l][r], rig.v_index)
    got_k, got_v = rig.host_pools()
    assert got_k.tobytes() == kp.tobytes()             # every byte: appended slots and nothing else
    assert got_v.tobytes() == vp.tobytes()
    # attention over the grown cache, last layer
    q = W.queries(seed + 1, geom, B)
    out = rig.decode(L - 1, q, table, model.ctx, running, sentinel=1.5)
    ref = oracle.decode_attn(q, model.K[L - 1], model.V[L - 1], model.ctx, running)
    got = to_f64(out)
    live = running == 1
    assert np.abs(got[live] - ref[live]).max() <= tol(geom)
    assert (got[~live] == 1.5).all()
    rig.close()


def test_position_past_the_table_row_writes_nothing_and_does_not_advance():
    geom = W.Geometry(1, 4, 4, 64, 16, 8, 2, "f32")
    rig = Rig(geom, 2)
    table = np.array([[0, 1], [2, 3]], dtype=np.int32)
    ctx = [32, 5]                                      # request 0 has filled its two blocks
    dev = rig.dev
    before_k, before_v = (x.copy() for x in rig.host_pools())
    kn, vn = _new_rows(5, geom, 2)
    td = torch.as_tensor(table, device=dev)
    cd = torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=dev)
    md = torch.ones(2, dtype=torch.uint8, device=dev)
    with torch.cuda.stream(rig.compute):
        rig.lamps.kv_append(0, 2, n2t(kn, dev), n2t(vn, dev), td, cd, md, True)
    rig.compute.synchronize()
    assert cd.cpu().tolist() == [32, 6]
    got_k, got_v = rig.host_pools()
    exp_k, exp_v = before_k.copy(), before_v.copy()
    exp_k[2, 0][:, 5 * 64:6 * 64] = kn[1]
    exp_v[2, 0][:, 5 * 64:6 * 64] = vn[1]
    assert got_k.tobytes() == exp_k.tobytes() and got_v.tobytes() == exp_v.tobytes()
    rig.close()


def test_append_rejects_bad_host_arguments():
    import paper_2410_18248_amd as P
    geom = W.Geometry(2, 4, 4, 64, 16, 8, 2, "f32")
    rig = Rig(geom, 2)
    x = torch.zeros(8, device=rig.dev)
    with pytest.raises(P.LampsError) as e:
        rig.lamps.kv_append(2, 1, x, x, x, x, x, True)
    assert e.value.status == -2
    with pytest.raises(P.LampsError) as e:
        rig.lamps.kv_append(0, 3, x, x, x, x, x, True)
    assert e.value.status == -2
    with pytest.raises(P.LampsError) as e:
        rig.lamps.kv_append(0, 1, None, x, x, x, x, True)
    assert e.value.status == -1
    rig.close()
