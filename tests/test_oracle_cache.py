"""Pins for the oracle's logical KV-cache model (Section 2.2.1: the cache grows
by one key and one value vector per layer per iteration) -- CPU only."""
import numpy as np

import lamps_workloads as W
from oracle import LogicalCache


def _start(seed, L, ctx, Hkv=2, D=8):
    g = W.Geometry(L, Hkv, Hkv, D, 16, 8, 4, "f32")
    K = [[W.logical_kv(seed + 7 * l + r, g, c)[0] for r, c in enumerate(ctx)] for l in range(L)]
    V = [[W.logical_kv(seed + 7 * l + r, g, c)[1] for r, c in enumerate(ctx)] for l in range(L)]
    return g, K, V


def test_iterations_stack_the_new_rows_in_order():
    ctx = [3, 0, 5]
    g, K, V = _start(11, 2, ctx)
    m = LogicalCache(2, ctx, K, V)
    news = []
    for it in range(4):
        step = []
        for l in range(2):
            kn = W.normal_f32(100 + 10 * it + l, 3 * 2 * 8).reshape(3, 2, 8)
            vn = W.normal_f32(200 + 10 * it + l, 3 * 2 * 8).reshape(3, 2, 8)
            m.append(l, kn, vn, [1, 1, 1], advance=(l == 1))
            step.append((kn, vn))
        news.append(step)
    assert m.ctx == [7, 4, 9]
    for l in range(2):
        for r in range(3):
            want_k = np.concatenate([K[l][r]] + [news[it][l][0][r][None] for it in range(4)])
            want_v = np.concatenate([V[l][r]] + [news[it][l][1][r][None] for it in range(4)])
            assert m.K[l][r].tobytes() == want_k.tobytes()
            assert m.V[l][r].tobytes() == want_v.tobytes()


def test_requests_outside_the_running_batch_append_nothing():
    ctx = [4, 6]
    g, K, V = _start(12, 1, ctx)
    m = LogicalCache(1, ctx, K, V)
    kn = np.full((2, 2, 8), 9.0, np.float32)
    m.append(0, kn, -kn, [0, 1], advance=True)
    assert m.ctx == [4, 7]
    assert m.K[0][0].tobytes() == K[0][0].tobytes() and m.V[0][0].tobytes() == V[0][0].tobytes()
    assert (m.K[0][1][6] == 9.0).all() and (m.V[0][1][6] == -9.0).all()
    assert m.K[0][1][:6].tobytes() == K[0][1].tobytes()


def test_without_advance_the_position_is_rewritten_not_extended():
    ctx = [2]
    g, K, V = _start(13, 1, ctx)
    m = LogicalCache(1, ctx, K, V)
    a = np.full((1, 2, 8), 1.0, np.float32)
    b = np.full((1, 2, 8), 2.0, np.float32)
    m.append(0, a, a, [1], advance=False)
    m.append(0, b, b, [1], advance=True)
    assert m.ctx == [3] and m.K[0][0].shape[0] == 3
    assert (m.K[0][0][2] == 2.0).all() and (m.V[0][0][2] == 2.0).all()


def test_model_copies_its_inputs():
    ctx = [2]
    g, K, V = _start(14, 1, ctx)
    m = LogicalCache(1, ctx, K, V)
    K[0][0][:] = 0
    assert (m.K[0][0] != 0).any()
