"""ctypes binding of include/tokencake_kv.h: same names, argument marshalling only.

Pointers may be given as ints, torch tensors (``data_ptr()``), numpy arrays or None; id arrays
must be int32 numpy arrays (host); streams may be ``torch.cuda.Stream``, a raw handle or None.
Functions return the library's status code unchanged unless noted; ``check(rc)`` raises.
"""
import ctypes
import os

import numpy as np

from . import build as _build

__all__ = [
    "TC_OK", "TC_ERR_INVAL", "TC_ERR_RANGE", "TC_ERR_DUP", "TC_ERR_SHARED", "TC_ERR_NOMEM",
    "TC_ERR_HOST_NOMEM", "TC_ERR_NOT_PINNED", "TC_ERR_HIP", "TC_ERR_LIMIT",
    "TC_NOALLOC_MAX_BLOCKS", "TC_NOALLOC_STAGING_BYTES", "tc_offload_noalloc",
    "TC_PATH_AUTO", "TC_PATH_DIRECT", "TC_PATH_DIRECT_IF_DUPLEX", "TC_PATH_STAGED",
    "tc_hbm_write", "tc_hbm_read", "tc_stage_on_device",
    "TcError", "check", "tc_pool_desc", "tc_opts", "tc_xfer_desc", "tc_stats_t", "library_path",
    "tc_create", "tc_destroy", "tc_record_bytes", "tc_strerror", "tc_alloc", "tc_alloc_at", "tc_ref",
    "tc_free", "tc_filter_private", "tc_host_alloc", "tc_host_free", "tc_offload", "tc_upload",
    "tc_offload_batch", "tc_upload_batch", "tc_poll", "tc_sync", "tc_stats", "tc_set_profiling",
    "tc_arena_base", "tc_copy_contiguous", "tc_copy_via_lds", "tc_hbm_stream", "tc_naive_transfer",
    "tc_cost_model", "tc_waiting_req", "tc_cost_fit", "tc_calibrate", "tc_estimate_transfer_ms",
    "tc_should_offload", "tc_upload_budget", "tc_gradual_reserve",
    "tc_req_state", "tc_lifecycle_step", "tc_forecaster_create", "tc_forecaster_destroy",
    "tc_forecaster_observe", "tc_forecaster_estimate",
    "tc_alloc_prefer", "TC_RES_ABSENT", "TC_RES_CPU", "TC_RES_H2D", "TC_FNV_BASIS", "tc_index_hit",
    "tc_index_create", "tc_index_destroy", "tc_index_insert", "tc_index_lookup", "tc_index_begin_upload",
    "tc_index_finish_upload", "tc_index_remove", "tc_index_pending", "tc_index_size",
    "tc_fnv1a64", "tc_chain_hashes",
    "TC_GATE_PASS", "TC_GATE_CPU_FULL", "TC_GATE_STALL_SHORT", "TC_GATE_NO_FIT", "TC_GATE_LOW_PRESSURE",
    "tc_gate_input", "tc_upload_cand", "tc_offload_gate", "tc_upload_plan",
]

TC_OK = 0
TC_ERR_INVAL, TC_ERR_RANGE, TC_ERR_DUP, TC_ERR_SHARED = -1, -2, -3, -4
TC_ERR_NOMEM, TC_ERR_HOST_NOMEM, TC_ERR_NOT_PINNED, TC_ERR_HIP, TC_ERR_LIMIT = -5, -6, -7, -8, -9
TC_NOALLOC_MAX_BLOCKS, TC_NOALLOC_STAGING_BYTES = 1024, 64 << 20
TC_PATH_AUTO, TC_PATH_DIRECT, TC_PATH_DIRECT_IF_DUPLEX, TC_PATH_STAGED = 0, 1, 2, 3
TC_RES_ABSENT, TC_RES_CPU, TC_RES_H2D = 0, 1, 2
TC_FNV_BASIS = 0xCBF29CE484222325
TC_GATE_PASS, TC_GATE_CPU_FULL, TC_GATE_STALL_SHORT, TC_GATE_NO_FIT, TC_GATE_LOW_PRESSURE = 0, 1, 2, 3, 4


class tc_pool_desc(ctypes.Structure):
    _fields_ = [
        ("kv_base", ctypes.c_void_p), ("scales", ctypes.c_void_p),
        ("num_layers", ctypes.c_uint32), ("num_blocks", ctypes.c_uint32),
        ("page_bytes", ctypes.c_uint32), ("block_size_tokens", ctypes.c_uint32),
        ("scales_per_block", ctypes.c_uint32),
    ]


class tc_opts(ctypes.Structure):
    _fields_ = [
        ("host_arena_bytes", ctypes.c_uint64), ("staging_bytes", ctypes.c_uint64),
        ("staging_slots", ctypes.c_uint32), ("max_grid", ctypes.c_uint32),
        ("direct_offload", ctypes.c_uint32), ("direct_upload", ctypes.c_uint32), ("direct_grid", ctypes.c_uint32),
        ("host_tail_div", ctypes.c_uint32), ("auto_direct_bytes", ctypes.c_uint64),
        ("overlap_kernels", ctypes.c_uint32), ("reserved0", ctypes.c_uint32),
    ]


class tc_xfer_desc(ctypes.Structure):
    _fields_ = [
        ("block_ids", ctypes.c_void_p), ("n", ctypes.c_uint32),
        ("host_buf", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
    ]


class tc_stats_t(ctypes.Structure):
    _fields_ = [
        ("gpu_blocks_total", ctypes.c_uint32), ("gpu_blocks_free", ctypes.c_uint32),
        ("gpu_blocks_used", ctypes.c_uint32), ("gpu_blocks_pending_free", ctypes.c_uint32),
        ("gpu_blocks_shared", ctypes.c_uint32), ("ops_in_flight", ctypes.c_uint32),
        ("host_slots_total", ctypes.c_uint64), ("host_slots_used", ctypes.c_uint64),
        ("n_offloads", ctypes.c_uint64), ("n_uploads", ctypes.c_uint64),
        ("blocks_offloaded", ctypes.c_uint64), ("blocks_uploaded", ctypes.c_uint64),
        ("bytes_offloaded", ctypes.c_uint64), ("bytes_uploaded", ctypes.c_uint64),
        ("gather_launches", ctypes.c_uint64), ("scatter_launches", ctypes.c_uint64),
        ("gather_bytes", ctypes.c_uint64), ("scatter_bytes", ctypes.c_uint64),
        ("gather_ms", ctypes.c_double), ("scatter_ms", ctypes.c_double),
        ("direct_launches", ctypes.c_uint64), ("direct_bytes", ctypes.c_uint64), ("direct_ms", ctypes.c_double),
        ("d2h_copies", ctypes.c_uint64), ("h2d_copies", ctypes.c_uint64),
        ("d2h_bytes", ctypes.c_uint64), ("h2d_bytes", ctypes.c_uint64),
        ("d2h_ms", ctypes.c_double), ("h2d_ms", ctypes.c_double),
        ("transfers_failed", ctypes.c_uint64),
        ("transfers_overlapped", ctypes.c_uint64),
    ]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class tc_cost_model(ctypes.Structure):
    _fields_ = [
        ("off_a_ms", ctypes.c_double), ("off_b_ms_per_block", ctypes.c_double),
        ("up_a_ms", ctypes.c_double), ("up_b_ms_per_block", ctypes.c_double),
    ]

    def as_tuple(self):
        return (self.off_a_ms, self.off_b_ms_per_block, self.up_a_ms, self.up_b_ms_per_block)


class tc_waiting_req(ctypes.Structure):
    _fields_ = [("kv_blocks", ctypes.c_uint32), ("work_tokens", ctypes.c_double)]


class tc_req_state(ctypes.Structure):
    _fields_ = [("state", ctypes.c_uint8), ("finish_seen", ctypes.c_uint8),
                ("copy_in_flight", ctypes.c_uint8), ("reserved", ctypes.c_uint8)]

    def as_tuple(self):
        return (self.state, bool(self.finish_seen), bool(self.copy_in_flight))


class tc_gate_input(ctypes.Structure):
    _fields_ = [("req_blocks", ctypes.c_uint32), ("cpu_free_blocks", ctypes.c_uint32),
                ("gpu_used_blocks", ctypes.c_uint32), ("gpu_total_blocks", ctypes.c_uint32),
                ("pressure_threshold", ctypes.c_double), ("t_fc_ms", ctypes.c_double),
                ("v_throughput_tokens_per_ms", ctypes.c_double)]


class tc_upload_cand(ctypes.Structure):
    _fields_ = [("importance", ctypes.c_double), ("urgency", ctypes.c_double), ("deficit", ctypes.c_uint32)]


class tc_index_hit(ctypes.Structure):
    _fields_ = [("key", ctypes.c_uint64), ("cpu_record", ctypes.c_void_p),
                ("gpu_block", ctypes.c_int32), ("state", ctypes.c_int32)]

    def as_tuple(self):
        return (self.key, self.state, self.cpu_record or 0, self.gpu_block)


class TcError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"tokencake_kv error {code}: {tc_strerror(code)}")
        self.code = code


def check(rc):
    if rc != TC_OK:
        raise TcError(rc)
    return rc


_lib = None


def library_path():
    return _build.LIB


def _load():
    """Loads the built library; builds it first only when none exists.  Never falls back."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    try:
        import torch  # noqa: F401  the process must share torch's HIP runtime, so it is loaded first
    except ImportError:
        pass
    lib = ctypes.CDLL(_build.LIB)
    vp, u32, u64, ci = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int
    sig = {
        "tc_create": (ci, [ctypes.POINTER(tc_pool_desc), ctypes.POINTER(tc_opts), ctypes.POINTER(vp)]),
        "tc_destroy": (ci, [vp]),
        "tc_record_bytes": (u64, [vp]),
        "tc_strerror": (ctypes.c_char_p, [ci]),
        "tc_alloc": (ci, [vp, u32, vp]),
        "tc_alloc_at": (ci, [vp, vp, u32]),
        "tc_ref": (ci, [vp, vp, u32]),
        "tc_free": (ci, [vp, vp, u32]),
        "tc_filter_private": (ci, [vp, vp, u32, vp, ctypes.POINTER(u32)]),
        "tc_host_alloc": (ci, [vp, u32, ctypes.POINTER(vp)]),
        "tc_host_free": (ci, [vp, vp]),
        "tc_offload": (ci, [vp, vp, u32, vp, vp]),
        "tc_upload": (ci, [vp, vp, vp, u32, vp, vp]),
        "tc_offload_noalloc": (ci, [ctypes.POINTER(tc_pool_desc), vp, u32, vp, vp]),
        "tc_offload_batch": (ci, [vp, ctypes.POINTER(tc_xfer_desc), u32, vp]),
        "tc_upload_batch": (ci, [vp, ctypes.POINTER(tc_xfer_desc), u32, vp]),
        "tc_poll": (ci, [vp]),
        "tc_sync": (ci, [vp]),
        "tc_stats": (ci, [vp, ctypes.POINTER(tc_stats_t)]),
        "tc_set_profiling": (ci, [vp, ci]),
        "tc_arena_base": (vp, [vp]),
        "tc_copy_contiguous": (ci, [vp, vp, u64, vp]),
        "tc_copy_via_lds": (ci, [vp, vp, u64, ci, vp]),
        "tc_hbm_write": (ci, [vp, u64, vp]),
        "tc_hbm_read": (ci, [vp, u64, vp]),
        "tc_stage_on_device": (ci, [vp, ci, vp, u32, vp, vp]),
        "tc_hbm_stream": (ci, [vp, vp, vp, u64, ctypes.c_float, u32, vp]),
        "tc_naive_transfer": (ci, [vp, vp, u32, vp, ci, ci, vp]),
        "tc_cost_fit": (ci, [vp, vp, vp, u32, ctypes.POINTER(tc_cost_model)]),
        "tc_calibrate": (ci, [vp, vp, u32, u32, vp, ctypes.POINTER(tc_cost_model)]),
        "tc_estimate_transfer_ms": (ctypes.c_double, [ctypes.POINTER(tc_cost_model), u32]),
        "tc_should_offload": (ci, [ctypes.POINTER(tc_cost_model), u32, ctypes.c_double, ctypes.c_double,
                                   ctypes.POINTER(tc_waiting_req), u32, ctypes.POINTER(ctypes.c_int32)]),
        "tc_upload_budget": (u32, [u32, u32, u32]),
        "tc_gradual_reserve": (u32, [u32, u32, u32]),
        "tc_lifecycle_step": (ci, [ctypes.POINTER(tc_req_state), ci, ctypes.POINTER(ci)]),
        "tc_forecaster_create": (ci, [ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.POINTER(vp)]),
        "tc_forecaster_destroy": (ci, [vp]),
        "tc_forecaster_observe": (ci, [vp, u32, ctypes.c_double]),
        "tc_forecaster_estimate": (ctypes.c_double, [vp, u32, ci, ctypes.c_double]),
        "tc_alloc_prefer": (ci, [vp, vp, u32, vp]),
        "tc_offload_gate": (ci, [ctypes.POINTER(tc_cost_model), ctypes.POINTER(tc_gate_input),
                                 ctypes.POINTER(tc_waiting_req), u32, ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ci)]),
        "tc_upload_plan": (ci, [ctypes.POINTER(tc_upload_cand), u32, u32, u32, u32, vp, vp]),
        "tc_index_create": (ci, [ctypes.POINTER(vp)]),
        "tc_index_destroy": (ci, [vp]),
        "tc_index_insert": (ci, [vp, vp, vp, vp, u64, u32]),
        "tc_index_lookup": (ci, [vp, vp, u32, ctypes.POINTER(tc_index_hit), ctypes.POINTER(u32)]),
        "tc_index_begin_upload": (ci, [vp, vp, vp, u32]),
        "tc_index_finish_upload": (ci, [vp, vp, u32]),
        "tc_index_remove": (ci, [vp, vp, u32]),
        "tc_index_pending": (u32, [vp, vp, u32]),
        "tc_index_size": (u64, [vp]),
        "tc_fnv1a64": (u64, [vp, u64, u64]),
        "tc_chain_hashes": (ci, [vp, u64, u32, u64, vp, ctypes.POINTER(u64)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


# ------------------------------------------------------------------ marshalling
def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, ctypes.c_void_p):
        return x.value
    raise TypeError(f"cannot take the address of {type(x).__name__}")


def _ids(ids):
    a = np.ascontiguousarray(ids, dtype=np.int32)
    return a, (a.ctypes.data if a.size else None), int(a.size)


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


# ------------------------------------------------------------------ the calls
def tc_create(kv_base, scales, num_layers, num_blocks, page_bytes, block_size_tokens, scales_per_block=0,
              host_arena_bytes=0, staging_bytes=0, staging_slots=0, max_grid=0, direct_offload=0, direct_upload=0, direct_grid=0,
              host_tail_div=0, auto_direct_bytes=0, overlap_kernels=0):
    """Returns (rc, ctx); ctx is an opaque handle (int) or None."""
    desc = tc_pool_desc(_ptr(kv_base), _ptr(scales), num_layers, num_blocks, page_bytes, block_size_tokens,
                        scales_per_block)
    opts = tc_opts(host_arena_bytes, staging_bytes, staging_slots, max_grid, direct_offload, direct_upload,
                   direct_grid, host_tail_div, auto_direct_bytes, overlap_kernels, 0)
    out = ctypes.c_void_p()
    rc = _load().tc_create(ctypes.byref(desc), ctypes.byref(opts), ctypes.byref(out))
    return rc, out.value


def tc_destroy(ctx):
    return _load().tc_destroy(ctx)


def tc_record_bytes(ctx):
    return int(_load().tc_record_bytes(ctx))


def tc_strerror(code):
    return _load().tc_strerror(code).decode()


def tc_alloc(ctx, n):
    """Returns (rc, ids) with ids an int32 numpy array (empty on failure)."""
    out = np.empty(n, dtype=np.int32)
    rc = _load().tc_alloc(ctx, n, out.ctypes.data if n else None)
    return rc, (out if rc == TC_OK else out[:0])


def tc_alloc_at(ctx, ids):
    a, p, n = _ids(ids)
    return _load().tc_alloc_at(ctx, p, n)


def tc_alloc_prefer(ctx, preferred):
    """Returns (rc, ids): preferred[i] where still free, a fresh block otherwise (empty on failure)."""
    a, p, n = _ids(preferred)
    out = np.empty(n, dtype=np.int32)
    rc = _load().tc_alloc_prefer(ctx, p, n, out.ctypes.data if n else None)
    return rc, (out if rc == TC_OK else out[:0])


def tc_ref(ctx, ids):
    a, p, n = _ids(ids)
    return _load().tc_ref(ctx, p, n)


def tc_free(ctx, ids):
    a, p, n = _ids(ids)
    return _load().tc_free(ctx, p, n)


def tc_filter_private(ctx, ids):
    """Returns (rc, private_ids)."""
    a, p, n = _ids(ids)
    out = np.empty(n, dtype=np.int32)
    m = ctypes.c_uint32(0)
    rc = _load().tc_filter_private(ctx, p, n, out.ctypes.data if n else None, ctypes.byref(m))
    return rc, out[: m.value].copy()


def tc_host_alloc(ctx, n_blocks):
    """Returns (rc, address) — address is an int, or None for n_blocks = 0 / failure."""
    out = ctypes.c_void_p()
    rc = _load().tc_host_alloc(ctx, n_blocks, ctypes.byref(out))
    return rc, out.value


def tc_host_free(ctx, host_buf):
    return _load().tc_host_free(ctx, _ptr(host_buf))


def tc_offload(ctx, block_ids, host_buf, stream=None):
    a, p, n = _ids(block_ids)
    return _load().tc_offload(ctx, p, n, _ptr(host_buf), _stream(stream))


def tc_upload(ctx, host_buf, new_block_ids, block_table=None, stream=None):
    a, p, n = _ids(new_block_ids)
    return _load().tc_upload(ctx, _ptr(host_buf), p, n, _ptr(block_table), _stream(stream))


def tc_offload_noalloc(kv_base, scales, num_layers, num_blocks, page_bytes, block_size_tokens, scales_per_block,
                       block_ids, host_buf, stream=None):
    desc = tc_pool_desc(_ptr(kv_base), _ptr(scales), num_layers, num_blocks, page_bytes, block_size_tokens,
                        scales_per_block)
    a, p, n = _ids(block_ids)
    return _load().tc_offload_noalloc(ctypes.byref(desc), p, n, _ptr(host_buf), _stream(stream))


def _descs(items):
    """items: iterable of (ids, host_buf[, block_table])."""
    keep = []
    arr = (tc_xfer_desc * len(items))()
    for i, it in enumerate(items):
        a, p, n = _ids(it[0])
        keep.append(a)
        arr[i] = tc_xfer_desc(p, n, _ptr(it[1]), _ptr(it[2]) if len(it) > 2 else None)
    return keep, arr


def tc_offload_batch(ctx, items, stream=None):
    keep, arr = _descs(items)
    return _load().tc_offload_batch(ctx, arr, len(items), _stream(stream))


def tc_upload_batch(ctx, items, stream=None):
    keep, arr = _descs(items)
    return _load().tc_upload_batch(ctx, arr, len(items), _stream(stream))


def tc_poll(ctx):
    return _load().tc_poll(ctx)


def tc_sync(ctx):
    return _load().tc_sync(ctx)


def tc_stats(ctx):
    """Returns (rc, tc_stats_t)."""
    st = tc_stats_t()
    rc = _load().tc_stats(ctx, ctypes.byref(st))
    return rc, st


def tc_set_profiling(ctx, on):
    return _load().tc_set_profiling(ctx, int(bool(on)))


def tc_arena_base(ctx):
    return _load().tc_arena_base(ctx)


def tc_copy_contiguous(dst, src, nbytes, stream=None):
    return _load().tc_copy_contiguous(_ptr(dst), _ptr(src), nbytes, _stream(stream))


def tc_copy_via_lds(dst, src, nbytes, lds_direct_loads=0, stream=None):
    return _load().tc_copy_via_lds(_ptr(dst), _ptr(src), nbytes, int(lds_direct_loads), _stream(stream))


def tc_hbm_write(dst, nbytes, stream=None):
    return _load().tc_hbm_write(_ptr(dst), nbytes, _stream(stream))


def tc_hbm_read(src, nbytes, stream=None):
    return _load().tc_hbm_read(_ptr(src), nbytes, _stream(stream))


def tc_stage_on_device(ctx, direction, block_ids, dev_records, stream=None):
    a, p, n = _ids(block_ids)
    return _load().tc_stage_on_device(ctx, direction, p, n, _ptr(dev_records), _stream(stream))


def tc_hbm_stream(a, b, c, n, s=0.5, iters=1, stream=None):
    return _load().tc_hbm_stream(_ptr(a), _ptr(b), _ptr(c), n, s, iters, _stream(stream))


def tc_naive_transfer(ctx, block_ids, host_buf, mode, direction, stream=None):
    a, p, n = _ids(block_ids)
    return _load().tc_naive_transfer(ctx, p, n, _ptr(host_buf), mode, direction, _stream(stream))


def _model(model):
    return model if isinstance(model, tc_cost_model) else tc_cost_model(*model)


def tc_cost_fit(n_blocks, offload_ms, upload_ms):
    """Returns (rc, tc_cost_model)."""
    n = np.ascontiguousarray(n_blocks, dtype=np.uint32)
    o = np.ascontiguousarray(offload_ms, dtype=np.float64)
    u = np.ascontiguousarray(upload_ms, dtype=np.float64)
    out = tc_cost_model()
    m = int(n.size) if n.size == o.size == u.size else 0
    rc = _load().tc_cost_fit(n.ctypes.data, o.ctypes.data, u.ctypes.data, m, ctypes.byref(out))
    return rc, out


def tc_calibrate(ctx, sizes, reps=3, stream=None):
    """Returns (rc, tc_cost_model) measured on this context."""
    n = np.ascontiguousarray(sizes, dtype=np.uint32)
    out = tc_cost_model()
    rc = _load().tc_calibrate(ctx, n.ctypes.data, int(n.size), reps, _stream(stream), ctypes.byref(out))
    return rc, out


def tc_estimate_transfer_ms(model, n_blocks):
    return float(_load().tc_estimate_transfer_ms(ctypes.byref(_model(model)), n_blocks))


def tc_should_offload(model, req_blocks, t_fc_ms, v_throughput_tokens_per_ms, waiting):
    """waiting: sequence of (kv_blocks, work_tokens).  Returns (rc, chosen index): rc 1 = offload, 0 = reject."""
    q = (tc_waiting_req * max(len(waiting), 1))()
    for i, (b, w) in enumerate(waiting):
        q[i] = tc_waiting_req(int(b), float(w))
    chosen = ctypes.c_int32(-1)
    rc = _load().tc_should_offload(ctypes.byref(_model(model)), req_blocks, t_fc_ms, v_throughput_tokens_per_ms,
                                   q, len(waiting), ctypes.byref(chosen))
    return rc, chosen.value


def tc_offload_gate(model, req_blocks, cpu_free_blocks, gpu_used_blocks, gpu_total_blocks, pressure_threshold,
                    t_fc_ms, v_throughput_tokens_per_ms, waiting):
    """Returns (rc, reason, chosen index): rc 1 = no hard rejection applies, 0 = rejected for `reason`."""
    q = (tc_waiting_req * max(len(waiting), 1))()
    for i, (b, w) in enumerate(waiting):
        q[i] = tc_waiting_req(int(b), float(w))
    gi = tc_gate_input(req_blocks, cpu_free_blocks, gpu_used_blocks, gpu_total_blocks, pressure_threshold,
                       t_fc_ms, v_throughput_tokens_per_ms)
    chosen, reason = ctypes.c_int32(-1), ctypes.c_int(-1)
    rc = _load().tc_offload_gate(ctypes.byref(_model(model)), ctypes.byref(gi), q, len(waiting),
                                 ctypes.byref(chosen), ctypes.byref(reason))
    return rc, reason.value, chosen.value


def tc_upload_plan(candidates, gpu_free, d_critical, shared_free):
    """candidates: sequence of (importance, urgency, deficit).  Returns (rc, order, reserve) as lists."""
    n = len(candidates)
    c = (tc_upload_cand * max(n, 1))()
    for i, (imp, urg, d) in enumerate(candidates):
        c[i] = tc_upload_cand(float(imp), float(urg), int(d))
    order = np.zeros(max(n, 1), dtype=np.uint32)
    reserve = np.zeros(max(n, 1), dtype=np.uint32)
    rc = _load().tc_upload_plan(c, n, gpu_free, d_critical, shared_free, order.ctypes.data, reserve.ctypes.data)
    return rc, [int(x) for x in order[:n]], [int(x) for x in reserve[:n]]


def tc_upload_budget(gpu_free, d_critical, shared_free):
    return int(_load().tc_upload_budget(gpu_free, d_critical, shared_free))


def tc_gradual_reserve(remain, deficit, budget):
    return int(_load().tc_gradual_reserve(remain, deficit, budget))


def tc_lifecycle_step(req, event):
    """req: tc_req_state (updated in place on success).  Returns (rc, action)."""
    action = ctypes.c_int(0)
    rc = _load().tc_lifecycle_step(ctypes.byref(req), event, ctypes.byref(action))
    return rc, action.value


def tc_forecaster_create(alpha, gamma, default_ms):
    """Returns (rc, handle)."""
    out = ctypes.c_void_p()
    rc = _load().tc_forecaster_create(alpha, gamma, default_ms, ctypes.byref(out))
    return rc, out.value


def tc_forecaster_destroy(f):
    return _load().tc_forecaster_destroy(f)


def tc_forecaster_observe(f, fn_type, elapsed_ms):
    return _load().tc_forecaster_observe(f, fn_type, elapsed_ms)


def tc_forecaster_estimate(f, fn_type, t_user_ms=None):
    return float(_load().tc_forecaster_estimate(f, fn_type, int(t_user_ms is not None), t_user_ms or 0.0))


def _keys(keys):
    a = np.ascontiguousarray(keys, dtype=np.uint64)
    return a, (a.ctypes.data if a.size else None), int(a.size)


def tc_index_create():
    """Returns (rc, handle)."""
    out = ctypes.c_void_p()
    rc = _load().tc_index_create(ctypes.byref(out))
    return rc, out.value


def tc_index_destroy(ix):
    return _load().tc_index_destroy(ix)


def tc_index_insert(ix, keys, gpu_blocks, host_buf, record_bytes):
    k, kp, n = _keys(keys)
    a, ap, m = _ids(gpu_blocks)
    if m != n:
        return TC_ERR_INVAL
    return _load().tc_index_insert(ix, kp, ap, _ptr(host_buf), record_bytes, n)


def tc_index_lookup(ix, keys):
    """Returns (rc, hits): hits is a list of (key, state, cpu_record, gpu_block) for the leading run present."""
    k, kp, n = _keys(keys)
    out = (tc_index_hit * max(n, 1))()
    hits = ctypes.c_uint32(0)
    rc = _load().tc_index_lookup(ix, kp, n, out, ctypes.byref(hits))
    return rc, [out[i].as_tuple() for i in range(hits.value)]


def tc_index_begin_upload(ix, keys, new_gpu_blocks):
    k, kp, n = _keys(keys)
    a, ap, m = _ids(new_gpu_blocks)
    if m != n:
        return TC_ERR_INVAL
    return _load().tc_index_begin_upload(ix, kp, ap, n)


def tc_index_finish_upload(ix, keys):
    k, kp, n = _keys(keys)
    return _load().tc_index_finish_upload(ix, kp, n)


def tc_index_remove(ix, keys):
    k, kp, n = _keys(keys)
    return _load().tc_index_remove(ix, kp, n)


def tc_index_pending(ix, keys):
    k, kp, n = _keys(keys)
    return int(_load().tc_index_pending(ix, kp, n))


def tc_index_size(ix):
    return int(_load().tc_index_size(ix))


def tc_fnv1a64(data, basis=TC_FNV_BASIS):
    b = bytes(data)
    return int(_load().tc_fnv1a64(ctypes.cast(ctypes.c_char_p(b), ctypes.c_void_p), len(b), basis))


def tc_chain_hashes(tokens, block_size, parent=0):
    """Returns (rc, keys) with keys a uint64 numpy array, one per whole block."""
    t = np.ascontiguousarray(tokens, dtype=np.int32)
    out = np.empty(int(t.size) // block_size if block_size else 0, dtype=np.uint64)
    n_out = ctypes.c_uint64(0)
    rc = _load().tc_chain_hashes(t.ctypes.data if t.size else None, int(t.size), block_size, parent,
                                 out.ctypes.data if out.size else None, ctypes.byref(n_out))
    return rc, out[: n_out.value]
