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


def test_page_unpage_round_trip_and_layout():
    g = W.Geometry(2, 4, 2, 8, 16, 10, 4, "f32")
    kp = np.full(g.pool_shape, np.nan, dtype=np.float32)
    k, _ = W.logical_kv(1, g, 37)
    row = np.array([6, 1, 9, -1], dtype=np.int32)
    W.page(kp, 1, row, k)
    np.testing.assert_array_equal(W.unpage(kp, 1, row, 37), k)
    # element (t, head, d) sits at pool[table[t // bs], layer, head, t % bs, d]
    for t, h, d in [(0, 0, 0), (16, 1, 3), (36, 0, 7)]:
        flat = ((((row[t // 16] * 2 + 1) * 2 + h) * 16 + t % 16) * 8 + d)
        assert kp.reshape(-1)[flat] == k[t, h, d]
    assert np.isnan(kp[9, 1, :, 5:, :]).all()        # tail slots untouched
    assert np.isnan(kp[:, 0]).all()                  # other layer untouched


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
    assert w3.ctx_lens.min() >= 4096 and w3.part_tokens * 8 <= w3.ctx_lens.min()
    nb = np.array([w3.geom.blocks_for(c) for c in w3.ctx_lens])
    assert nb[w3.state == W.SWAP].sum() >= 0.4 * nb.sum()
    w4 = W.workload(4)
    assert w4.batch == 512 and w4.ctx_lens.min() >= 64 and w4.ctx_lens.max() <= 4096
    assert [(w4.state == s).sum() for s in (W.PRESERVE, W.DISCARD, W.SWAP)] == [19, 19, 39]
    pool_gb = 2 * w4.geom.num_blocks * w4.geom.block_half_bytes / 1e9
    assert pool_gb < 0.85 * 288
