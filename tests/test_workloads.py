"""The seeded input generators and the pager -- CPU only."""
import numpy as np
import torch

import lamps_workloads as W


def test_splitmix64_published_vectors():
    # first outputs of the reference splitmix64 for seeds 0 and 1234567
    assert [int(x) for x in W.splitmix64(0, 3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4,
                                                    0x06C45D188009454F]
    assert [int(x) for x in W.splitmix64(1234567, 2)] == [6457827717110365317,
                                                          3203168211198807973]


def test_normal_moments_and_reproducibility():
    z = W.normal_f32(5, 200000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    np.testing.assert_array_equal(z[:1000], W.normal_f32(5, 1000))


def test_permutation_is_a_permutation():
    p = W.permutation(3, 1000)
    assert sorted(p.tolist()) == list(range(1000)) and (p != np.arange(1000)).sum() > 900


def test_bf16_rounding_matches_torch():
    x = np.concatenate([W.normal_f32(8, 5000), np.array([0.0, -0.0, 1.00390625, 1.01171875, 3e38],
                                                        dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(W.f32_to_bf16_bits(x), want)
    np.testing.assert_array_equal(W.bf16_bits_to_f32(want),
                                  torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_page_unpage_round_trip_and_plain_layout():
    g = W.Geometry(2, 4, 4, 8, 16, 10, 4, "f32")
    assert g.kv_layout == "plain"
    k_index, v_index = g.tile_index_maps()
    kp = np.full(g.pool_shape, np.nan, dtype=np.float32)
    k, _ = W.logical_kv(1, g, 37)
    row = np.array([6, 1, 9, -1], dtype=np.int32)
    W.page(kp, 1, row, k, k_index)
    np.testing.assert_array_equal(W.unpage(kp, 1, row, 37, k_index), k)
    # element (t, head, d) sits at pool[table[t // bs], layer, head][(t % bs) * D + d]
    for t, h, d in [(0, 0, 0), (16, 1, 3), (36, 3, 7)]:
        flat = ((((row[t // 16] * 2 + 1) * 4 + h) * 16 + t % 16) * 8 + d)
        assert kp.reshape(-1)[flat] == k[t, h, d]
    assert np.isnan(kp[9, 1].reshape(4, 16, 8)[:, 5:, :]).all()    # tail slots untouched
    assert np.isnan(kp[:, 0]).all()                                   # other layer untouched


def test_tiled_layout_is_a_permutation_with_the_documented_runs():
    g = W.Geometry(1, 8, 2, 128, 32, 4, 2, "bf16")
    assert g.kv_layout == "tiled" and W.Geometry(1, 8, 8, 128, 32, 4, 2, "bf16").kv_layout == "plain"
    k_index, v_index = g.tile_index_maps()
    for m in (k_index, v_index):                       # a bijection onto the tile
        assert sorted(m.ravel().tolist()) == list(range(32 * 128))
    # keys: the 8 dims d..d+7 (d % 8 == 0) of one slot are one 16-byte run; the 16 slots of a
    # sub-tile follow each other for a fixed group of 8 dims
    assert (np.diff(k_index[5, 40:48]) == 1).all() and k_index[5, 40] % 8 == 0
    assert k_index[6, 40] - k_index[5, 40] == 8 and k_index[21, 40] - k_index[5, 40] == 16 * 128
    # values: 4 consecutive slots of one dim are adjacent; then the same slots of dim + 16
    assert (np.diff(v_index[8:12, 3]) == 1).all() and v_index[8, 3] % 4 == 0
    assert v_index[8, 19] - v_index[8, 3] == 4 and v_index[8, 4] - v_index[8, 3] == 8
    assert v_index[8, 35] - v_index[8, 3] == 4 * 16 * 8          # next pair of 16-dim slabs
    # round trip through the pager
    kp = np.zeros(g.pool_shape, dtype=np.uint16)
    vp = np.zeros(g.pool_shape, dtype=np.uint16)
    k, v = W.logical_kv(3, g, 45)
    row = np.array([2, 0], dtype=np.int32)
    W.page(kp, 0, row, k, k_index)
    W.page(vp, 0, row, v, v_index)
    np.testing.assert_array_equal(W.unpage(kp, 0, row, 45, k_index), k)
    np.testing.assert_array_equal(W.unpage(vp, 0, row, 45, v_index), v)


def test_configurations_have_the_stated_shape():
    w0 = W.workload(0)
    assert w0.ctx_lens.tolist() == [17, 64, 130, 200] and w0.state[2] == W.SWAP
    assert sum(w0.geom.blocks_for(c) for c in w0.ctx_lens) == 28
    w1 = W.workload(1)
    assert w1.batch == 64 and 128 <= w1.ctx_lens.min() and w1.ctx_lens.max() <= 2048
    assert (w1.state == W.PRESERVE).sum() == 6 and (w1.state == W.SWAP).sum() == 7
    w2 = W.workload(2)
    assert w2.batch == 256 and w2.ctx_lens.min() >= 32 and w2.ctx_lens.max() <= 8192
    assert 700 < np.median(w2.ctx_lens) < 1400 and (w2.state == W.SWAP).sum() == 26
    w3 = W.workload(3)
    assert w3.ctx_lens.min() >= 4096
    nb = np.array([w3.geom.blocks_for(c) for c in w3.ctx_lens])
    assert nb[w3.state == W.SWAP].sum() >= 0.4 * nb.sum()
    w4 = W.workload(4)
    assert w4.batch == 512 and w4.ctx_lens.min() >= 64 and w4.ctx_lens.max() <= 4096
    assert [(w4.state == s).sum() for s in (W.PRESERVE, W.DISCARD, W.SWAP)] == [19, 19, 39]
    pool_gb = 2 * w4.geom.num_blocks * w4.geom.block_half_bytes / 1e9
    assert pool_gb < 0.85 * 288
