"""ctypes front end of ``lamps_oracle.c`` (test infrastructure, see package doc).

Arrays are numpy: ``float32`` for fp32 data, ``uint16`` holding bf16 bit
patterns for bf16 data.  The result is always float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lamps_oracle.c")
_LIB = os.path.join(_HERE, "liblamps_oracle.so")
_lib = None

F32, BF16 = 0, 1


_SANITIZE = os.environ.get("LAMPS_SANITIZE", "") not in ("", "0")
if _SANITIZE:                                   # the sanitizer build lives apart from the normal one
    _LIB = os.path.join(os.path.dirname(_HERE), "_build", "sanitize", "liblamps_oracle.so")


def build(force=False):
    """Compile the C oracle with gcc (plain -O2, OpenMP for the (r,h) loop).  With
    LAMPS_SANITIZE=1: with clang, AddressSanitizer and UndefinedBehaviorSanitizer, one thread."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        if _SANITIZE:
            os.makedirs(os.path.dirname(_LIB), exist_ok=True)
            subprocess.check_call(
                ["/opt/rocm/lib/llvm/bin/clang", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
                 "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                 "-shared-libasan", "-fno-omit-frame-pointer", "-o", _LIB, _SRC, "-lm"])
        else:
            subprocess.check_call(
                ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                 "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.lamps_oracle_decode_attn.restype = ctypes.c_int
        lib.lamps_oracle_decode_attn.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_double, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p),
            ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int]
        lib.lamps_oracle_widen.restype = ctypes.c_double
        lib.lamps_oracle_widen.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int]
        lib.lamps_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle takes float32 or uint16 (bf16 bits), got %s" % a.dtype)


def max_threads():
    return int(_load().lamps_oracle_max_threads())


def widen(a, i):
    """Element i of a float32 / bf16-bits array as the double the oracle uses."""
    a = np.ascontiguousarray(a)
    return float(_load().lamps_oracle_widen(a.ctypes.data, int(i), _code(a)))


def decode_attn(q, K, V, ctx_lens, running, scale=None, out=None, threads=1):
    """One layer of one decode iteration (Section 2.2 equation; Algorithm 1's
    running batch decides which rows are computed).

    q        [B][H][D]
    K, V     lists of length B; K[r] is the logical sequence [C_r][H_kv][D]
             (None allowed for paused requests / empty contexts)
    ctx_lens [B] ints, running [B] truthy = in the running batch
    out      optional float64 [B][H][D]; rows of paused requests keep their
             contents (a fresh array is NaN-filled so misuse is visible)
    """
    lib = _load()
    q = np.ascontiguousarray(q)
    B, H, D = q.shape
    code = _code(q)
    ctx = np.ascontiguousarray(np.asarray(ctx_lens, dtype=np.int32))
    run = np.ascontiguousarray(np.asarray(running).astype(np.uint8))
    assert ctx.shape == (B,) and run.shape == (B,)
    Hkv = None
    keep = []
    kp = (ctypes.c_void_p * B)()
    vp = (ctypes.c_void_p * B)()
    for r in range(B):
        if not run[r] or ctx[r] == 0:
            continue
        k = np.ascontiguousarray(K[r])
        v = np.ascontiguousarray(V[r])
        assert _code(k) == code and _code(v) == code
        assert k.shape == v.shape and k.ndim == 3 and k.shape[2] == D
        assert k.shape[0] >= ctx[r], "logical sequence shorter than ctx_len"
        if Hkv is None:
            Hkv = k.shape[1]
        assert k.shape[1] == Hkv
        keep += [k, v]
        kp[r] = k.ctypes.data
        vp[r] = v.ctypes.data
    if Hkv is None:
        Hkv = H
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    if out is None:
        out = np.full((B, H, D), np.nan, dtype=np.float64)
    assert out.dtype == np.float64 and out.shape == (B, H, D) and out.flags.c_contiguous
    rc = lib.lamps_oracle_decode_attn(code, B, H, Hkv, D, float(scale), q.ctypes.data, kp, vp,
                                      ctx.ctypes.data, run.ctypes.data, out.ctypes.data,
                                      int(threads))
    if rc != 0:
        raise RuntimeError("lamps_oracle_decode_attn failed (rc=%d)" % rc)
    return out


def prefill_attn(q, K, V, q_start, ctx_lens, scale=None, threads=1):
    """Attention for several new tokens per request at once (the recompute of a
    discarded context, a prompt, an API response): the Section 2.2 equation for
    each new token over the cached positions up to and including its own.

    q        [total][H][D], the new tokens of request r are rows
             q_start[r] .. q_start[r+1]-1 and sit at the LAST positions of its
             sequence: row q_start[r]+i is position ctx_lens[r] - n_r + i
    K, V     lists; K[r] is the logical sequence [ctx_lens[r]][H_kv][D], new
             tokens included
    Returns float64 [total][H][D].  Every row is an independent evaluation of
    the decode equation with its own context length."""
    q = np.ascontiguousarray(q)
    Ks, Vs, ctx = [], [], []
    for r in range(len(ctx_lens)):
        n = int(q_start[r + 1]) - int(q_start[r])
        assert 0 <= n <= int(ctx_lens[r])
        k, v = np.ascontiguousarray(K[r]), np.ascontiguousarray(V[r])
        for i in range(n):
            Ks.append(k)
            Vs.append(v)
            ctx.append(int(ctx_lens[r]) - n + i + 1)
    assert len(ctx) == q.shape[0] == int(q_start[len(ctx_lens)])
    if not ctx:
        return np.zeros(q.shape, dtype=np.float64)
    return decode_attn(q, Ks, Vs, ctx, np.ones(len(ctx), dtype=np.uint8), scale=scale, threads=threads)
