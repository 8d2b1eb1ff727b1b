"""Pins for the CPU oracle's attention (Section 2.2 equation) -- CPU only."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
from attn_pins import ALL, NON_BRUTE, as_f64


def oracle_attn(q, K, V, ctx, running, scale=None, out=None):
    return oracle.decode_attn(q, K, V, ctx, running, scale=scale, out=out)


@pytest.mark.parametrize("check", ALL, ids=lambda c: c.__name__)
def test_oracle_passes_pin(check):
    check(oracle_attn)


def test_threads_do_not_change_result():
    g = W.Geometry(1, 8, 4, 32, 16, 1, 1, "bf16")
    ctx = [100, 3, 57, 1, 64]
    q = W.queries(5, g, 5)
    KV = [W.logical_kv(9 + r, g, c) for r, c in enumerate(ctx)]
    K, V = [k for k, _ in KV], [v for _, v in KV]
    a = oracle.decode_attn(q, K, V, ctx, [1] * 5, threads=1)
    b = oracle.decode_attn(q, K, V, ctx, [1] * 5, threads=4)
    np.testing.assert_array_equal(a, b)


def test_bf16_widening_is_exact():
    bits = np.array([0x0000, 0x8000, 0x3F80, 0xBF80, 0x4049, 0x0001, 0x7F7F, 0x0080, 0x3DCD],
                    dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.widen(bits, i) for i in range(len(bits))])
    np.testing.assert_array_equal(got, want)
    f = np.array([1.5, -2.25e-30, 3.4e38], dtype=np.float32)
    np.testing.assert_array_equal([oracle.widen(f, i) for i in range(3)], f.astype(np.float64))


# ---- planted mistakes: each must be rejected by the battery ------------------
def _reference(q, K, V, ctx, running, scale=None, out=None, *, mistake=None):
    """A numpy copy of the definition in which one mistake can be planted."""
    B, H, D = q.shape
    Hkv = next((k.shape[1] for k, c in zip(K, ctx) if k is not None and c > 0), H)
    G = H // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    if mistake == "no_scale":
        scale = 1.0
    if out is None:
        out = np.full((B, H, D), np.nan)
    qf = as_f64(q)
    for r in range(B):
        if not running[r] and mistake != "writes_paused":
            continue
        C = int(ctx[r])
        if mistake == "ctx_minus_one":
            C = max(C - 1, 1) if C > 0 else 0
        if mistake == "ctx_plus_one" and K[r] is not None:
            C = min(C + 1, K[r].shape[0])
        for h in range(H):
            if C == 0 or K[r] is None:
                out[r, h] = 0.0
                continue
            g = h // G
            if mistake == "gqa_modulo":
                g = h % Hkv
            k = as_f64(K[r][:C, g])
            v = as_f64(V[r][:C, (Hkv - 1 - g) if mistake == "wrong_v_head" else g])
            s = (k @ qf[r, h]) * scale
            if mistake == "sign":
                s = -s
            if mistake == "score_uses_v":
                s = (v @ qf[r, h]) * scale
            p = np.exp(s - s.max())
            if mistake == "unnormalised":
                out[r, h] = p @ v
            elif mistake == "mean_norm":
                out[r, h] = (p @ v) / C
            else:
                out[r, h] = (p @ v) / p.sum()
    return out


def _run(checks, fn):
    for c in checks:
        try:
            c(fn)
        except AssertionError:
            return False
    return True


def test_unplanted_copy_passes():
    assert _run(ALL, _reference)


@pytest.mark.parametrize("mistake", ["no_scale", "ctx_minus_one", "ctx_plus_one", "gqa_modulo",
                                      "wrong_v_head", "sign", "score_uses_v", "unnormalised",
                                      "mean_norm", "writes_paused"])
def test_planted_mistake_is_caught(mistake):
    def fn(*a, **k):
        return _reference(*a, mistake=mistake, **k)
    assert not _run(ALL, fn), "battery accepted a wrong implementation: " + mistake
    # the pins that do not re-type the formula catch it on their own
    assert not _run(NON_BRUTE, fn), "only brute force caught: " + mistake


# ---------------------------------------------------------------- several new tokens at once
def _causal_torch(q, K, V, n_new):
    """softmax(mask(q K^T / sqrt(D))) V in float64 with torch, new tokens last."""
    import torch
    C, Hkv, D = K.shape
    H = q.shape[1]
    G = H // Hkv
    qt = torch.from_numpy(q.astype(np.float64))                       # [n][H][D]
    Kt = torch.from_numpy(K.astype(np.float64)).repeat_interleave(G, dim=1)   # [C][H][D]
    Vt = torch.from_numpy(V.astype(np.float64)).repeat_interleave(G, dim=1)
    s = torch.einsum("nhd,chd->hnc", qt, Kt) / np.sqrt(D)
    pos = torch.arange(C - n_new, C)[:, None]
    s = s.masked_fill(torch.arange(C)[None, :] > pos, float("-inf"))
    return torch.einsum("hnc,chd->nhd", torch.softmax(s, dim=-1), Vt).numpy()


def test_prefill_equals_masked_dense_attention_in_torch():
    import oracle
    g = W.Geometry(1, 4, 2, 16, 16, 8, 8, "f32")
    ctx, new = [37, 5, 20], [9, 5, 1]
    K, V = zip(*[W.logical_kv(70 + r, g, c) for r, c in enumerate(ctx)])
    q_start = np.concatenate([[0], np.cumsum(new)])
    q = W.queries(71, g, int(q_start[-1]))
    got = oracle.prefill_attn(q, K, V, q_start, ctx)
    for r in range(3):
        want = _causal_torch(q[q_start[r]:q_start[r + 1]], K[r], V[r], new[r])
        assert np.abs(got[q_start[r]:q_start[r + 1]] - want).max() < 1e-12


def test_prefill_rows_are_decode_steps_and_first_token_sees_only_itself():
    import oracle
    g = W.Geometry(1, 2, 2, 8, 16, 8, 8, "f32")
    K, V = W.logical_kv(80, g, 12)
    q = W.queries(81, g, 12)
    full = oracle.prefill_attn(q, [K], [V], [0, 12], [12])            # the whole sequence is new
    assert np.array_equal(full[0], V[0].astype(np.float64))           # position 0: softmax over one key
    last = oracle.decode_attn(q[11:12], [K], [V], [12], [1])
    assert np.array_equal(full[11], last[0])
    tail = oracle.prefill_attn(q[8:], [K], [V], [0, 4], [12])         # only the last four are new
    assert np.array_equal(tail, full[8:])
