"""The battery of pins that an implementation of the Section 2.2 attention
equation must pass.  It is a function of the implementation so that the same
battery can be shown to reject implementations with a planted mistake
(test_oracle_attention.py plants them in numpy copies, on the CPU)."""
import os

import numpy as np
import torch

import lamps_workloads as W

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def as_f64(a):
    if a.dtype == np.uint16:
        return W.bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def draw(seed, B, H, Hkv, D, ctx, dtype):
    g = W.Geometry(1, H, Hkv, D, 16, 1, 1, dtype)
    q = W.queries(seed, g, B)
    K, V = [], []
    for r, c in enumerate(ctx):
        k, v = W.logical_kv(seed + 17 * (r + 1), g, c)
        K.append(k)
        V.append(v)
    return q, K, V


def brute_force(q, K, V, ctx, running, scale=None):
    """Second, independently written evaluation: one dense padded score matrix
    per kv-head group, -inf mask, NO max subtraction (safe in fp64 for O(1)
    scores), explicit normalisation, dense matmul."""
    B, H, D = q.shape
    Hkv = next(k.shape[1] for k, c in zip(K, ctx) if k is not None and c > 0)
    G = H // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    T = max(int(c) for c in ctx)
    out = np.full((B, H, D), np.nan)
    qf = as_f64(q)
    for r in range(B):
        if not running[r]:
            continue
        if ctx[r] == 0:
            out[r] = 0.0
            continue
        kf = np.zeros((T, Hkv, D))
        vf = np.zeros((T, Hkv, D))
        kf[:ctx[r]] = as_f64(K[r][:ctx[r]])
        vf[:ctx[r]] = as_f64(V[r][:ctx[r]])
        for g in range(Hkv):
            S = qf[r, g * G:(g + 1) * G] @ kf[:, g, :].T * scale          # [G][T]
            S[:, ctx[r]:] = -np.inf
            E = np.exp(S)
            out[r, g * G:(g + 1) * G] = (E @ vf[:, g, :]) / E.sum(axis=1, keepdims=True)
    return out


def check_brute_force(attn):
    cases = [(11, 3, 4, 4, 8, [5, 1, 33], "f32"), (12, 4, 8, 2, 16, [17, 64, 3, 40], "f32"),
             (13, 2, 6, 3, 8, [9, 30], "bf16"), (14, 3, 4, 1, 32, [2, 16, 31], "bf16")]
    for seed, B, H, Hkv, D, ctx, dt in cases:
        q, K, V = draw(seed, B, H, Hkv, D, ctx, dt)
        run = np.ones(B, dtype=np.uint8)
        got = attn(q, K, V, ctx, run)
        ref = brute_force(q, K, V, ctx, run)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def check_torch_library(attn):
    """Reduces to torch.softmax(q K^T / sqrt(D)) V in float64, head by head."""
    for seed, H, Hkv, D, C, dt in [(21, 4, 4, 16, 37, "f32"), (22, 8, 2, 8, 50, "bf16")]:
        q, K, V = draw(seed, 1, H, Hkv, D, [C], dt)
        got = attn(q, K, V, [C], [1])
        G = H // Hkv
        tq = torch.from_numpy(as_f64(q))[0]
        tk = torch.from_numpy(as_f64(K[0]))
        tv = torch.from_numpy(as_f64(V[0]))
        for h in range(H):
            w = torch.softmax(tq[h] @ tk[:, h // G, :].T / np.sqrt(D), dim=-1)
            np.testing.assert_allclose(got[0, h], (w @ tv[:, h // G, :]).numpy(), rtol=0, atol=1e-12)


def check_golden_sigmoid(attn):
    want = np.loadtxt(os.path.join(GOLD, "sigmoid_two_tokens.txt"))
    q = np.array([[[2, 0, 0, 0]]], dtype=np.float32)
    K = [np.array([[[0, 0, 0, 0]], [[1, 0, 0, 0]]], dtype=np.float32)]
    V = [np.array([[[1, 0, 0, 0]], [[0, 1, 0, 0]]], dtype=np.float32)]
    got = attn(q, K, V, [2], [1])
    np.testing.assert_allclose(got[0, 0], want, rtol=0, atol=1e-15)


def check_closed_forms(attn):
    H, Hkv, D, C = 4, 2, 8, 23
    q, K, V = draw(31, 1, H, Hkv, D, [C], "f32")
    G = H // Hkv
    # one cached position: output is that value row exactly
    got = attn(q, K, V, [1], [1])
    for h in range(H):
        np.testing.assert_array_equal(got[0, h], V[0][0, h // G].astype(np.float64))
    # all key rows equal: uniform weights, output is the mean value row
    Keq = [np.repeat(K[0][:1], C, axis=0)]
    got = attn(q, Keq, V, [C], [1])
    for h in range(H):
        np.testing.assert_allclose(got[0, h], V[0][:, h // G].astype(np.float64).mean(0), atol=1e-13)
    # zero query: uniform weights
    got = attn(np.zeros_like(q), K, V, [C], [1])
    for h in range(H):
        np.testing.assert_allclose(got[0, h], V[0][:, h // G].astype(np.float64).mean(0), atol=1e-13)
    # constant value rows: output is that constant whatever the keys
    Vc = [np.broadcast_to(np.float32(0.625), V[0].shape).copy()]
    got = attn(q, K, Vc, [C], [1])
    np.testing.assert_allclose(got, 0.625, atol=1e-14)
    # one key strongly aligned with the query: output tends to its value row
    Kd = [K[0].copy()]
    t0 = 7
    for g in range(Hkv):
        Kd[0][t0, g] = 40.0 * q[0, g * G]          # aligned with the group's first head
    got = attn(q, Kd, V, [C], [1])
    for g in range(Hkv):
        np.testing.assert_allclose(got[0, g * G], V[0][t0, g].astype(np.float64), atol=1e-9)
    # empty context of a running request: empty weighted sum
    got = attn(q, [None], [None], [0], [1])
    np.testing.assert_array_equal(got, 0.0)


def check_invariants(attn):
    B, H, Hkv, D = 2, 6, 2, 16
    ctx = [29, 12]
    q, K, V = draw(41, B, H, Hkv, D, ctx, "f32")
    run = [1, 1]
    base = attn(q, K, V, ctx, run)
    # joint permutation of the cached positions
    Kp, Vp = [], []
    for r in range(B):
        p = W.permutation(99 + r, ctx[r])
        Kp.append(K[r][p])
        Vp.append(V[r][p])
    np.testing.assert_allclose(attn(q, Kp, Vp, ctx, run), base, atol=1e-13)
    # the same vector added to every key row of a request shifts all its scores equally
    u = W.normal_f32(7, D).astype(np.float32) * np.float32(0.25)
    Ks = [(k.astype(np.float64) + u).astype(np.float32) for k in K]
    ref_shift = brute_force(q, Ks, V, ctx, run)     # fp32 re-rounding of K+u changes values slightly
    np.testing.assert_allclose(attn(q, Ks, V, ctx, run), ref_shift, atol=1e-12)
    Kexact = [np.round(k * 8) / 8 for k in K]       # multiples of 1/8: shift below is exact
    ue = (np.round(u * 8) / 8).astype(np.float32)
    qe = (np.round(q * 8) / 8).astype(np.float32)
    a = attn(qe, [k.astype(np.float32) for k in Kexact], V, ctx, run)
    b = attn(qe, [(k + ue).astype(np.float32) for k in Kexact], V, ctx, run)
    np.testing.assert_allclose(a, b, atol=1e-12)
    # value scaling and the convex hull of the value rows
    Vs = [(-4.0 * v).astype(np.float32) for v in V]   # power of two: exact in fp32
    np.testing.assert_allclose(attn(q, K, Vs, ctx, run), -4.0 * base, atol=1e-12)
    G = H // Hkv
    for r in range(B):
        for h in range(H):
            vv = V[r][:ctx[r], h // G].astype(np.float64)
            assert np.all(base[r, h] <= vv.max(0) + 1e-12) and np.all(base[r, h] >= vv.min(0) - 1e-12)
    # only the first ctx_len positions count: NaN beyond them changes nothing
    Kn = [np.concatenate([k, np.full((3,) + k.shape[1:], np.nan, np.float32)]) for k in K]
    Vn = [np.concatenate([v, np.full((3,) + v.shape[1:], np.nan, np.float32)]) for v in V]
    np.testing.assert_array_equal(attn(q, Kn, Vn, ctx, run), base)


def check_gqa_is_repeated_mha(attn):
    B, H, Hkv, D = 2, 8, 2, 8
    ctx = [19, 6]
    q, K, V = draw(51, B, H, Hkv, D, ctx, "bf16")
    G = H // Hkv
    got = attn(q, K, V, ctx, [1, 1])
    Kr = [np.repeat(k, G, axis=1) for k in K]       # each kv head G times, consecutively
    Vr = [np.repeat(v, G, axis=1) for v in V]
    np.testing.assert_array_equal(attn(q, Kr, Vr, ctx, [1, 1]), got)
    # distinct kv heads give distinct outputs, equal kv heads and equal queries the same
    q2 = q.copy()
    q2[:, 1] = q2[:, 0]
    got2 = attn(q2, K, V, ctx, [1, 1])
    np.testing.assert_array_equal(got2[:, 1], got2[:, 0])          # same group, same query
    q3 = q.copy()
    q3[:, G] = q3[:, 0]
    got3 = attn(q3, K, V, ctx, [1, 1])
    assert np.abs(got3[:, G] - got3[:, 0]).max() > 1e-3            # different group


def check_paused_rows_untouched(attn):
    B, H, Hkv, D = 3, 4, 4, 8
    ctx = [5, 9, 7]
    q, K, V = draw(61, B, H, Hkv, D, ctx, "f32")
    full = attn(q, K, V, ctx, [1, 1, 1])
    out = np.full((B, H, D), 12345.0)
    got = attn(q, [K[0], None, K[2]], [V[0], None, V[2]], ctx, [1, 0, 1], out=out)
    np.testing.assert_array_equal(got[1], 12345.0)
    np.testing.assert_array_equal(got[0], full[0])
    np.testing.assert_array_equal(got[2], full[2])


def check_scale_argument(attn):
    q, K, V = draw(71, 1, 2, 2, 8, [13], "f32")
    a = attn(q, K, V, [13], [1], scale=0.3)
    b = brute_force(q, K, V, [13], [1], scale=0.3)
    np.testing.assert_allclose(a, b, atol=1e-12)


ALL = [check_brute_force, check_torch_library, check_golden_sigmoid, check_closed_forms,
       check_invariants, check_gqa_is_repeated_mha, check_paused_rows_untouched,
       check_scale_argument]
# pins that do not re-derive the formula (closed forms, printed values, invariants, library)
NON_BRUTE = [c for c in ALL if c not in (check_brute_force, check_scale_argument)]
