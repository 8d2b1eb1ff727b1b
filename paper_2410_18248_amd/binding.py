"""ctypes binding of liblamps.so -- argument marshalling only.

Pointers may be given as ints, ctypes pointers, or objects with ``data_ptr()``
(torch tensors).  Nothing here computes: every step of the path runs in the
library's kernels, and there is no fallback if the library is missing.
"""
import ctypes
import os

LAMPS_F32, LAMPS_BF16 = 0, 1
LAMPS_LAYOUT_PLAIN, LAMPS_LAYOUT_TILED = 0, 1

STATUS = {0: "LAMPS_OK", -1: "LAMPS_ERR_INVALID", -2: "LAMPS_ERR_RANGE", -3: "LAMPS_ERR_DUP",
          -4: "LAMPS_ERR_DOUBLE_FREE", -5: "LAMPS_ERR_BUSY", -6: "LAMPS_ERR_NOMEM",
          -7: "LAMPS_ERR_HIP"}
LAMPS_ERR_BUSY = -5

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


class LampsError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("%s: %s" % (STATUS.get(status, status), text))
        self.status = status


class LampsConfig(ctypes.Structure):
    """Mirror of ``lamps_config``."""
    _fields_ = [("num_layers", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32),
                ("max_blocks_per_req", ctypes.c_int32), ("max_batch", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("part_tokens", ctypes.c_int32), ("staging_bytes", ctypes.c_int64),
                ("direct_copy_bytes", ctypes.c_int64), ("zero_copy_workgroups", ctypes.c_int32),
                ("max_swaps_in_flight", ctypes.c_int32)]


def lib_path():
    """The built library; LAMPS_LIBRARY overrides the in-tree path (to compare builds), and
    LAMPS_SANITIZE=1 selects the sanitizer build of the host code (CPU container only)."""
    if os.environ.get("LAMPS_LIBRARY"):
        return os.environ["LAMPS_LIBRARY"]
    if os.environ.get("LAMPS_SANITIZE", "") not in ("", "0"):
        return os.path.join(os.path.dirname(_HERE), "_build", "sanitize", "liblamps.so")
    return os.path.join(_HERE, "liblamps.so")


def load_library():
    """Loads liblamps.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if os.environ.get("LAMPS_SANITIZE", "") in ("", "0"):
        try:
            # torch bundles its own HIP runtime under the same soname as /opt/rocm's; whichever is
            # loaded first serves the whole process, and it has to be the one torch was built with
            import torch  # noqa: F401
        except ImportError:
            pass
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("liblamps.so is not built: run `python -m paper_2410_18248_amd.build`")
    lib = ctypes.CDLL(path)
    vp, i32, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64
    cfgp = ctypes.POINTER(LampsConfig)
    for name in ("lamps_kv_bytes_per_token", "lamps_block_bytes", "lamps_pool_bytes",
                 "lamps_workspace_bytes"):
        getattr(lib, name).restype = ctypes.c_size_t
        getattr(lib, name).argtypes = [cfgp]
    lib.lamps_kv_layout.restype = ctypes.c_int
    lib.lamps_kv_layout.argtypes = [cfgp]
    sig = {
        "lamps_create": [cfgp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)],
        "lamps_destroy": [vp],
        "lamps_decode_attn": [vp, i32, i32, vp, vp, vp, vp, vp],
        "lamps_decode_attn_static": [cfgp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp],
        "lamps_validate_args": [vp, i32, vp, vp, vp, vp],
        "lamps_kv_append": [vp, i32, i32, vp, vp, vp, vp, vp, i32],
        "lamps_kv_append_tokens": [vp, i32, i32, i32, vp, vp, vp, vp, vp],
        "lamps_prefill_attn": [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp],
        "lamps_swap_out": [vp, vp, i32, vp, ctypes.POINTER(u64)],
        "lamps_swap_in": [vp, vp, vp, i32, ctypes.POINTER(u64)],
        "lamps_swap_out_layered": [vp, vp, i32, vp, ctypes.POINTER(u64)],
        "lamps_swap_in_layered": [vp, vp, vp, i32, ctypes.POINTER(u64)],
        "lamps_compute_wait_layer": [vp, u64, i32],
        "lamps_set_swap_fence": [vp, i32],
        "lamps_swap_wait_compute": [vp],
        "lamps_ticket_query": [vp, u64],
        "lamps_ticket_wait": [vp, u64],
        "lamps_compute_wait": [vp, u64],
        "lamps_compute_wait_blocks": [vp, vp, i32],
        "lamps_alloc_blocks": [vp, i32, vp],
        "lamps_free_blocks": [vp, vp, i32],
        "lamps_num_free": [vp],
    }
    for name, args in sig.items():
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = args
    _sched_signatures(lib)
    lib.lamps_last_error.restype = ctypes.c_char_p
    lib.lamps_last_error.argtypes = [vp]
    _lib = lib
    return lib


# ---------------------------------------------------------------- scheduler (lamps_sched.h)
LAMPS_PRESERVE, LAMPS_DISCARD, LAMPS_SWAP, LAMPS_HANDLING_AUTO = 0, 1, 2, -1
LAMPS_POLICY_FCFS, LAMPS_POLICY_SJF, LAMPS_POLICY_SJF_TOTAL, LAMPS_POLICY_LAMPS, LAMPS_POLICY_FIXED = range(5)


class LampsCostModel(ctypes.Structure):
    _fields_ = [("it_a", ctypes.c_double), ("it_b", ctypes.c_double), ("fwd_a", ctypes.c_double),
                ("fwd_b", ctypes.c_double), ("sw_a", ctypes.c_double), ("sw_b", ctypes.c_double),
                ("swap_stalls", ctypes.c_int32), ("unit", ctypes.c_int32)]


class LampsSchedConfig(ctypes.Structure):
    _fields_ = [("policy", ctypes.c_int32), ("max_batch", ctypes.c_int32),
                ("memory_tokens", ctypes.c_int64), ("starvation_threshold", ctypes.c_int32),
                ("score_refresh", ctypes.c_int32), ("recompute_chunk", ctypes.c_int64),
                ("c_other", ctypes.c_double), ("bytes_per_token", ctypes.c_double),
                ("cost", LampsCostModel)]


class LampsSegment(ctypes.Structure):
    _fields_ = [("n_out", ctypes.c_int32), ("api_duration", ctypes.c_double),
                ("api_response", ctypes.c_int32), ("handling", ctypes.c_int32)]


class LampsBatchEntry(ctypes.Structure):
    _fields_ = [("id", ctypes.c_int64), ("swap_in", ctypes.c_int64), ("recompute", ctypes.c_int64),
                ("context", ctypes.c_int64)]


class LampsSchedEvent(ctypes.Structure):
    _fields_ = [("id", ctypes.c_int64), ("what", ctypes.c_int32), ("handling", ctypes.c_int32),
                ("context", ctypes.c_int64)]


def _sched_signatures(lib):
    d, i32, i64, vp = ctypes.c_double, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    P = ctypes.POINTER
    for name, args in (("lamps_waste_preserve", [d, d, d]), ("lamps_waste_discard", [d, d, d, d]),
                       ("lamps_waste_swap", [d, d, d]),
                       ("lamps_memory_over_time", [ctypes.c_int, i64, i64, d, i64, i64, d, d, d]),
                       ("lamps_sched_now", [vp])):
        getattr(lib, name).restype = d
        getattr(lib, name).argtypes = args
    for name, args in (("lamps_handling_strategy", [d, d, d, d, d, d]),
                       ("lamps_sched_create", [P(LampsSchedConfig), P(vp)]),
                       ("lamps_sched_destroy", [vp]),
                       ("lamps_sched_add", [vp, i64, d, i32, P(LampsSegment), i32, d]),
                       ("lamps_sched_next_batch", [vp, P(LampsBatchEntry), i32, P(i32)]),
                       ("lamps_sched_commit", [vp, d, P(LampsSchedEvent), i32, P(i32)]),
                       ("lamps_sched_take_discards", [vp, P(i64), i32, P(i32)]),
                       ("lamps_sched_run", [vp]),
                       ("lamps_sched_result", [vp, i64, P(d), P(d), P(i32), i32]),
                       ("lamps_sched_stats", [vp, P(i64), P(i64), P(i64)])):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = args


class LampsSched:
    """One ``lamps_sched``.  Methods carry the C names without the prefix."""

    def __init__(self, cfg):
        self.lib = load_library()
        self.cfg = cfg
        h = ctypes.c_void_p()
        rc = self.lib.lamps_sched_create(ctypes.byref(cfg), ctypes.byref(h))
        if rc != 0:
            raise LampsError(rc, "lamps_sched_create")
        self.h = h
        self._batch = (LampsBatchEntry * cfg.max_batch)()
        self._events = (LampsSchedEvent * cfg.max_batch)()

    def _check(self, rc, what):
        if rc < 0:
            raise LampsError(rc, what)
        return rc

    def destroy(self):
        if self.h:
            self.lib.lamps_sched_destroy(self.h)
            self.h = None

    def add(self, rid, arrival, prompt_tokens, segments, priority=0.0):
        """segments: [(n_out, api_duration or None, api_response, handling or None), ...]"""
        arr = (LampsSegment * len(segments))()
        for k, sg in enumerate(segments):
            n_out, api, rho = sg[0], sg[1], sg[2]
            h = sg[3] if len(sg) > 3 and sg[3] is not None else LAMPS_HANDLING_AUTO
            arr[k] = LampsSegment(n_out, -1.0 if api is None else api, rho, h)
        self._check(self.lib.lamps_sched_add(self.h, rid, arrival, prompt_tokens, arr, len(segments),
                                             priority), "lamps_sched_add")

    def next_batch(self):
        n = ctypes.c_int32()
        self._check(self.lib.lamps_sched_next_batch(self.h, self._batch, len(self._batch),
                                                    ctypes.byref(n)), "lamps_sched_next_batch")
        return [(b.id, b.swap_in, b.recompute, b.context) for b in self._batch[:n.value]]

    def commit(self, iteration_time=-1.0):
        n = ctypes.c_int32()
        self._check(self.lib.lamps_sched_commit(self.h, iteration_time, self._events,
                                                len(self._events), ctypes.byref(n)), "lamps_sched_commit")
        return [(e.id, e.what, e.handling, e.context) for e in self._events[:n.value]]

    def take_discards(self):
        out = []
        buf = (ctypes.c_int64 * 64)()
        while True:
            n = ctypes.c_int32()
            self._check(self.lib.lamps_sched_take_discards(self.h, buf, 64, ctypes.byref(n)),
                        "lamps_sched_take_discards")
            out += list(buf[:n.value])
            if n.value < 64:
                return out

    def run(self):
        self._check(self.lib.lamps_sched_run(self.h), "lamps_sched_run")

    def now(self):
        return self.lib.lamps_sched_now(self.h)

    def result(self, rid, n_segments=1):
        c, f = ctypes.c_double(), ctypes.c_double()
        h = (ctypes.c_int32 * max(n_segments, 1))()
        self._check(self.lib.lamps_sched_result(self.h, rid, ctypes.byref(c), ctypes.byref(f), h,
                                                n_segments), "lamps_sched_result")
        return c.value, f.value, list(h[:n_segments])

    def stats(self):
        a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        self._check(self.lib.lamps_sched_stats(self.h, ctypes.byref(a), ctypes.byref(b),
                                               ctypes.byref(c)), "lamps_sched_stats")
        return a.value, b.value, c.value


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):            # numpy array
        return x.ctypes.data
    return ctypes.cast(x, ctypes.c_void_p).value


def _ids(block_ids):
    ids = list(block_ids)
    return (ctypes.c_int32 * max(len(ids), 1))(*ids), len(ids)


def lamps_kv_bytes_per_token(cfg):
    return load_library().lamps_kv_bytes_per_token(ctypes.byref(cfg))


def lamps_kv_layout(cfg):
    return load_library().lamps_kv_layout(ctypes.byref(cfg))


def lamps_block_bytes(cfg):
    return load_library().lamps_block_bytes(ctypes.byref(cfg))


def lamps_pool_bytes(cfg):
    return load_library().lamps_pool_bytes(ctypes.byref(cfg))


def lamps_workspace_bytes(cfg):
    return load_library().lamps_workspace_bytes(ctypes.byref(cfg))


def lamps_decode_attn_static(cfg, compute_stream, layer, batch, q, k_pool, v_pool, block_table, ctx_lens,
                             running_mask, out):
    lib = load_library()
    rc = lib.lamps_decode_attn_static(ctypes.byref(cfg), compute_stream or None, layer, batch, _ptr(q),
                                      _ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(ctx_lens),
                                      _ptr(running_mask), _ptr(out))
    if rc < 0:
        raise LampsError(rc, lib.lamps_last_error(None).decode())


class Lamps:
    """One ``lamps_ctx``.  Methods carry the C names without the prefix."""

    def __init__(self, cfg, k_pool, v_pool, workspace, compute_stream=0, swap_out_stream=0,
                 swap_in_stream=0):
        self.lib = load_library()
        self.cfg = cfg
        self._keep = (k_pool, v_pool, workspace)     # the caller's memory must outlive the context
        h = ctypes.c_void_p()
        rc = self.lib.lamps_create(ctypes.byref(cfg), _ptr(k_pool), _ptr(v_pool), _ptr(workspace),
                                   compute_stream or None, swap_out_stream or None,
                                   swap_in_stream or None, ctypes.byref(h))
        if rc != 0:
            raise LampsError(rc, self.lib.lamps_last_error(None).decode())
        self.h = h

    def _check(self, rc):
        if rc < 0:
            raise LampsError(rc, self.lib.lamps_last_error(self.h).decode())
        return rc

    def destroy(self):
        if self.h:
            rc = self.lib.lamps_destroy(self.h)
            self.h = None
            if rc < 0:
                raise LampsError(rc, "lamps_destroy")

    def decode_attn(self, layer, batch, q, block_table, ctx_lens, running_mask, out):
        self._check(self.lib.lamps_decode_attn(self.h, layer, batch, _ptr(q), _ptr(block_table),
                                               _ptr(ctx_lens), _ptr(running_mask), _ptr(out)))

    def validate_args(self, batch, block_table, ctx_lens, running_mask):
        """Returns (bad requests, lowest bad request, reason, value); raises nothing for bad arguments."""
        rep = (ctypes.c_int32 * 4)()
        rc = self.lib.lamps_validate_args(self.h, batch, _ptr(block_table), _ptr(ctx_lens), _ptr(running_mask), rep)
        if rc < 0 and rc != -2:
            self._check(rc)
        if rc == -2 and rep[0] == 0:
            self._check(rc)                              # batch out of range
        return tuple(rep)

    def kv_append(self, layer, batch, k_new, v_new, block_table, ctx_lens, running_mask, advance):
        self._check(self.lib.lamps_kv_append(self.h, layer, batch, _ptr(k_new), _ptr(v_new),
                                             _ptr(block_table), _ptr(ctx_lens), _ptr(running_mask),
                                             1 if advance else 0))

    def kv_append_tokens(self, layer, n_req, total_tokens, k_new, v_new, q_start, block_table, ctx_lens):
        self._check(self.lib.lamps_kv_append_tokens(self.h, layer, n_req, total_tokens, _ptr(k_new),
                                                    _ptr(v_new), _ptr(q_start), _ptr(block_table),
                                                    _ptr(ctx_lens)))

    def prefill_attn(self, layer, n_req, total_tokens, q, q_start, block_table, ctx_lens, out,
                     max_new_tokens=0):
        self._check(self.lib.lamps_prefill_attn(self.h, layer, n_req, total_tokens, max_new_tokens, _ptr(q),
                                                _ptr(q_start), _ptr(block_table), _ptr(ctx_lens),
                                                _ptr(out)))

    def swap_out(self, block_ids, host_buf, layered=False):
        arr, n = _ids(block_ids)
        t = ctypes.c_uint64()
        f = self.lib.lamps_swap_out_layered if layered else self.lib.lamps_swap_out
        self._check(f(self.h, arr, n, _ptr(host_buf), ctypes.byref(t)))
        return t.value

    def swap_in(self, host_buf, block_ids, layered=False):
        arr, n = _ids(block_ids)
        t = ctypes.c_uint64()
        f = self.lib.lamps_swap_in_layered if layered else self.lib.lamps_swap_in
        self._check(f(self.h, _ptr(host_buf), arr, n, ctypes.byref(t)))
        return t.value

    def compute_wait_layer(self, ticket, layer):
        self._check(self.lib.lamps_compute_wait_layer(self.h, ticket, layer))

    def set_swap_fence(self, enabled):
        self._check(self.lib.lamps_set_swap_fence(self.h, 1 if enabled else 0))

    def swap_wait_compute(self):
        self._check(self.lib.lamps_swap_wait_compute(self.h))

    def ticket_query(self, ticket):
        rc = self.lib.lamps_ticket_query(self.h, ticket)
        if rc == LAMPS_ERR_BUSY:
            return False
        self._check(rc)
        return True

    def ticket_wait(self, ticket):
        self._check(self.lib.lamps_ticket_wait(self.h, ticket))

    def compute_wait(self, ticket):
        self._check(self.lib.lamps_compute_wait(self.h, ticket))

    def compute_wait_blocks(self, block_ids):
        arr, n = _ids(block_ids)
        self._check(self.lib.lamps_compute_wait_blocks(self.h, arr, n))

    def alloc_blocks(self, n):
        arr = (ctypes.c_int32 * max(n, 1))()
        self._check(self.lib.lamps_alloc_blocks(self.h, n, arr))
        return list(arr[:n])

    def free_blocks(self, block_ids):
        arr, n = _ids(block_ids)
        self._check(self.lib.lamps_free_blocks(self.h, arr, n))

    def num_free(self):
        return self._check(self.lib.lamps_num_free(self.h))

    def last_error(self):
        return self.lib.lamps_last_error(self.h).decode()
