"""Pins for the oracle's block-pool model (handling strategies of Section 1 /
Section 4.2) and the KV-bytes-per-token formula (Section 2.2.1) -- CPU only."""
import os
import zlib

import numpy as np
import pytest

import lamps_workloads as W
from oracle import AllocatorModel, PoolModel, kv_bytes_per_token

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _pool(seed, nb, half):
    b = W.splitmix64(seed, nb * half * 2 // 8 + 1).view(np.uint8)[:nb * half * 2]
    return PoolModel(b[:nb * half].reshape(nb, half), b[nb * half:].reshape(nb, half))


def _crc(row):
    return zlib.crc32(row.tobytes())


def test_kv_bytes_formula_matches_paper_example():
    L, Hkv, D, s, tokens, quoted_gb = np.loadtxt(os.path.join(GOLD, "kv_cache_size.txt"))
    total = kv_bytes_per_token(int(L), int(Hkv), int(D), int(s)) * int(tokens)
    assert total == 2 * 96 * 12288 * 2 * 512
    # "around 2.3 GB": 2.25 GiB / 2.42e9 B
    assert abs(total / 2 ** 30 - quoted_gb) / quoted_gb < 0.05
    assert abs(total / 1e9 - quoted_gb) / quoted_gb < 0.06


def test_swap_out_image_layout_and_pool_unchanged():
    p = _pool(1, 12, 40)
    k0, v0 = p.k.copy(), p.v.copy()
    ids = [7, 2, 11]
    host = p.swap_out(ids)
    assert host.shape == (3, 80)
    for i, b in enumerate(ids):                      # image = key bytes then value bytes
        assert host[i, :40].tobytes() == k0[b].tobytes()
        assert host[i, 40:].tobytes() == v0[b].tobytes()
    np.testing.assert_array_equal(p.k, k0)
    np.testing.assert_array_equal(p.v, v0)


def test_swap_round_trip_is_identity_and_touches_nothing_else():
    p = _pool(2, 16, 64)
    before_k = [_crc(r) for r in p.k]
    before_v = [_crc(r) for r in p.v]
    src = [3, 9, 4]
    dst = [12, 0, 15]                                # restored into different blocks
    want_k = p.k[src].copy()
    want_v = p.v[src].copy()
    host = p.swap_out(src)
    p.k[src] = 0xAB                                  # freed blocks get overwritten meanwhile
    p.v[src] = 0xCD
    p.swap_in(host, dst)
    np.testing.assert_array_equal(p.k[dst], want_k)
    np.testing.assert_array_equal(p.v[dst], want_v)
    for b in range(16):
        if b not in src and b not in dst:
            assert _crc(p.k[b]) == before_k[b] and _crc(p.v[b]) == before_v[b]


def test_layer_major_image_is_a_permutation_of_the_block_major_one():
    """Pins the layer-major image by the block-major one (itself pinned above): byte x of
    layer l of block i's key half sits at [l][i][0][x]; a reload of all layers is the same
    identity, a reload of the first layers only restores exactly those bytes."""
    L, lb = 3, 8
    p = _pool(4, 10, L * lb)
    src, dst = [5, 1, 8], [0, 9, 2]
    flat = p.swap_out(src)
    img = p.swap_out_layered(src, L)
    assert img.shape == (L, 3, 2, lb) and img.size == flat.size
    for i in range(3):
        for layer in range(L):
            assert img[layer, i, 0].tobytes() == flat[i, layer * lb:(layer + 1) * lb].tobytes()
            assert img[layer, i, 1].tobytes() == flat[i, L * lb + layer * lb:L * lb + (layer + 1) * lb].tobytes()
    q = PoolModel(p.k, p.v)
    q.swap_in(flat, dst)
    r = PoolModel(p.k, p.v)
    r.swap_in_layered(img, dst, L)
    np.testing.assert_array_equal(q.k, r.k)
    np.testing.assert_array_equal(q.v, r.v)
    part = PoolModel(p.k, p.v)
    part.swap_in_layered(img, dst, L, layers=[0])
    np.testing.assert_array_equal(part.k[dst][:, :lb], q.k[dst][:, :lb])
    np.testing.assert_array_equal(part.k[dst][:, lb:], p.k[dst][:, lb:])      # later layers not there yet
    np.testing.assert_array_equal(part.v[dst][:, lb:], p.v[dst][:, lb:])


def test_swap_in_rejects_duplicate_destination():
    p = _pool(3, 4, 8)
    with pytest.raises(AssertionError):
        p.swap_in(p.swap_out([0, 1]), [2, 2])


def test_allocator_lifo_and_conservation():
    a = AllocatorModel(8)
    assert a.alloc(3) == [0, 1, 2]
    assert a.alloc(2) == [3, 4]
    a.free([1, 3])
    assert a.num_free + len(a.live) == 8
    assert a.alloc(3) == [3, 1, 5]                   # last freed first, then fresh ids
    assert a.num_free + len(a.live) == 8
    with pytest.raises(ValueError):
        a.free([6])                                  # never allocated
    with pytest.raises(ValueError):
        a.free([0, 0])
    with pytest.raises(IndexError):
        a.free([8])
    with pytest.raises(MemoryError):
        a.alloc(3)
    assert a.num_free == 2 and sorted(a.live) == [0, 1, 2, 3, 4, 5]   # errors changed nothing


def test_free_count_per_handling_strategy():
    """Section 4.2: Preserve keeps memory constant; Discard and Swap bring it to
    zero during the call; swap-in restores it."""
    a = AllocatorModel(32)
    req = a.alloc(9)
    base = a.num_free
    assert a.num_free == base                        # Preserve: nothing changes
    a.free(req)                                      # Discard, or Swap after its copy
    assert a.num_free == base + 9
    back = a.alloc(9)                                # API returns
    assert a.num_free == base and len(back) == 9
