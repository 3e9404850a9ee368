"""ctypes binding of libpipemax.so: the same names as include/pipemax.h, argument marshalling only.

Importing this module loads the library and raises if it has not been built
(`python -m paper_2605_02189_amd.build`): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpipemax.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_02189_amd.build`")


def _preload_torch_hip_runtime():
    """Device pointers and streams handed to the library come from PyTorch, so both must live in ONE
    HIP runtime.  The PyTorch wheel ships its own libamdhip64 / libhsa-runtime64; loading them (by
    path, without importing torch) before libpipemax.so makes the dynamic loader resolve the
    library's HIP dependency to that same copy, whatever the import order."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.submodule_search_locations:
        return
    libdir = os.path.join(list(spec.submodule_search_locations)[0], "lib")
    for name in ("libhsa-runtime64.so", "libamdhip64.so"):
        path = os.path.join(libdir, name)
        if os.path.exists(path):
            C.CDLL(path, mode=C.RTLD_GLOBAL)


_preload_torch_hip_runtime()
_lib = C.CDLL(LIB_PATH)

OK, ERR_ARG, ERR_OOM_DEVICE, ERR_OOM_HOST = 0, -1, -2, -3
ERR_NOT_RESIDENT, ERR_POOL_EXHAUSTED, ERR_HIP, ERR_STATE = -4, -5, -6, -7
F32, BF16 = 0, 1
W_QKV, W_O, W_GU, W_D, G_ATTN, G_FFN = range(6)
FLAG_FORCE_GENERIC, FLAG_CAPTURE_LAYERS, FLAG_TIME_KERNELS, FLAG_NO_WRITEBACK = 1, 2, 4, 8
FLAG_TIME_ATTN_ONLY = 16
FLAG_STREAM_ORDERED_EVICT = 32
FLAG_DEVICE_LAYER_MAJOR = 64
K_CLASSES = ["norm", "gemm_qkv", "rope_append", "attn", "attn_merge", "gemm_o", "gemm_gu", "swiglu",
             "gemm_d", "misc"]
N_KCLASS = len(K_CLASSES)
HOST, INFLIGHT, GPU = 0, 1, 2

# every symbol include/pipemax.h declares
SYMBOLS = [
    "pipemax_stage_create", "pipemax_stage_destroy", "pipemax_set_weight", "pipemax_mb_define",
    "pipemax_mb_define_alias", "pipemax_mb_alias_of",
    "pipemax_kv_host_write", "pipemax_kv_host_read", "pipemax_kv_dev_read", "pipemax_prefetch_kv",
    "pipemax_decode_step", "pipemax_decode_step_noalloc", "pipemax_decode_step_seqs", "pipemax_prefill", "pipemax_evict_kv", "pipemax_sync", "pipemax_get_stats",
    "pipemax_reset_stats", "pipemax_set_flags", "pipemax_probe_copy", "pipemax_probe_read", "pipemax_probe_link",
    "pipemax_probe_link_strided", "pipemax_probe_launch", "pipemax_get_config", "pipemax_mb_size",
    "pipemax_get_ctx_lens", "pipemax_get_residency", "pipemax_get_block_table",
    "pipemax_get_layer_outputs", "pipemax_debug_fill_free_gpu_pages", "pipemax_debug_set_delays",
    "pipemax_last_error", "pipemax_version", "pipemax_page_elem_offset",
    "pipemax_plan_copy_runs", "pipemax_plan_gemm_splits", "pipemax_plan_attention_chunks", "pipemax_pool_create", "pipemax_pool_destroy", "pipemax_pool_alloc",
    "pipemax_pool_free", "pipemax_pool_free_count",
]
# every symbol include/pipemax_xfer.h declares
XFER_SYMBOLS = [
    "pipemax_xfer_create", "pipemax_xfer_destroy", "pipemax_xfer_submit", "pipemax_xfer_wait", "pipemax_xfer_poll",
    "pipemax_xfer_stream_wait", "pipemax_xfer_drain", "pipemax_xfer_get_stats", "pipemax_xfer_reset_stats",
    "pipemax_xfer_get_log", "pipemax_xfer_debug_set_host_us_per_mib", "pipemax_xfer_debug_pause",
    "pipemax_stage_attach_xfer",
]
XFER_URGENT, XFER_BULK, XFER_H2D, XFER_D2H = 0, 1, 0, 1
# every symbol include/pipemax_sched.h declares
SCHED_SYMBOLS = [
    "pipemax_sched_create", "pipemax_sched_destroy", "pipemax_sched_predict", "pipemax_sched_budget",
    "pipemax_sched_observe", "pipemax_sched_short_first_fill", "pipemax_sched_greedy_fill",
    "pipemax_sched_refine", "pipemax_sched_partition", "pipemax_sched_set_batch",
    "pipemax_sched_set_gpu_pages_free", "pipemax_sched_attach", "pipemax_sched_plan", "pipemax_sched_iterate",
]


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32),
                ("page_tokens", C.c_int32), ("n_microbatches", C.c_int32),
                ("max_seqs_per_mb", C.c_int32), ("max_ctx", C.c_int32),
                ("gpu_kv_bytes", C.c_uint64), ("host_kv_bytes", C.c_uint64),
                ("device", C.c_int32), ("flags", C.c_uint32),
                ("host_reserve_tokens", C.c_int32), ("wb_layers_per_copy", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("steps", C.c_uint64), ("tokens", C.c_uint64),
                ("h2d_bytes", C.c_uint64), ("h2d_copies", C.c_uint64),
                ("d2h_bytes", C.c_uint64), ("d2h_copies", C.c_uint64),
                ("table_uploads", C.c_uint64), ("relayout_jobs", C.c_uint64),
                ("host_enqueue_s", C.c_double), ("host_wait_s", C.c_double),
                ("h2d_ms", C.c_double), ("d2h_ms", C.c_double),
                ("kernel_ms", C.c_double * N_KCLASS), ("kernel_launches", C.c_uint64 * N_KCLASS),
                ("engine", C.c_int32), ("gpu_pages_total", C.c_int32), ("gpu_pages_free", C.c_int32),
                ("host_pages_total", C.c_int32), ("host_pages_free", C.c_int32),
                ("page_bytes", C.c_uint64), ("prefetch_stall_ms", C.c_double), ("prefetch_stalls", C.c_uint64)]

    def as_dict(self):
        d = {n: getattr(self, n) for n, _ in self._fields_ if n not in ("kernel_ms", "kernel_launches")}
        d["kernel_ms"] = {k: self.kernel_ms[i] for i, k in enumerate(K_CLASSES)}
        d["kernel_launches"] = {k: self.kernel_launches[i] for i, k in enumerate(K_CLASSES)}
        return d


_vp, _i32p = C.c_void_p, C.POINTER(C.c_int32)


class LinkProbe(C.Structure):
    _fields_ = [("h2d_s", C.c_double), ("d2h_s", C.c_double), ("wall_s", C.c_double),
                ("h2d_bytes", C.c_uint64), ("d2h_bytes", C.c_uint64), ("pieces", C.c_uint64)]


class LaunchProbe(C.Structure):
    _fields_ = [("host_enqueue_s", C.c_double), ("gpu_s", C.c_double), ("kernels", C.c_uint64)]


class XferConfig(C.Structure):
    _fields_ = [("device", C.c_int32), ("max_inflight_bulk", C.c_int32), ("chunk_bytes", C.c_uint64),
                ("log_capacity", C.c_int32), ("reserved", C.c_int32)]


class XferStats(C.Structure):
    _fields_ = [("requests", C.c_uint64 * 2), ("bytes", C.c_uint64 * 2), ("chunks", C.c_uint64 * 2),
                ("latency_sum_s", C.c_double * 2), ("latency_max_s", C.c_double * 2)]


class XferLog(C.Structure):
    _fields_ = [("ticket", C.c_uint64), ("offset", C.c_uint64), ("bytes", C.c_uint64), ("kind", C.c_int32),
                ("dir", C.c_int32)]


class SchedConfig(C.Structure):
    _fields_ = [("alpha_s", C.c_double), ("beta_s", C.c_double), ("delta_s", C.c_double),
                ("link_tokens_per_s", C.c_double), ("steady_rel_range", C.c_double),
                ("refine_tol_s", C.c_double), ("static_budget_tokens", C.c_int64),
                ("window", C.c_int32), ("max_refine_steps", C.c_int32), ("n_batches", C.c_int32),
                ("page_tokens", C.c_int32)]


class SchedIter(C.Structure):
    _fields_ = [("exec_batch", C.c_int32), ("n_exec", C.c_int32), ("prefetch_batch", C.c_int32),
                ("n_prefetch", C.c_int32), ("evict_batch", C.c_int32), ("n_evict", C.c_int32),
                ("steady", C.c_int32), ("n_exchanges", C.c_int32), ("budget_tokens", C.c_int64),
                ("prefetch_tokens", C.c_int64), ("gpu_pages_free", C.c_int64), ("t_hat_s", C.c_double),
                ("gap_s", C.c_double)]


_sig = {
    "pipemax_xfer_create": (C.c_int, [C.POINTER(XferConfig), C.POINTER(C.c_void_p)]),
    "pipemax_xfer_destroy": (C.c_int, [C.c_void_p]),
    "pipemax_xfer_submit": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t,
                                      C.POINTER(C.c_uint64)]),
    "pipemax_xfer_wait": (C.c_int, [C.c_void_p, C.c_uint64]),
    "pipemax_xfer_poll": (C.c_int, [C.c_void_p, C.c_uint64]),
    "pipemax_xfer_stream_wait": (C.c_int, [C.c_void_p, C.c_uint64, C.c_void_p]),
    "pipemax_xfer_drain": (C.c_int, [C.c_void_p]),
    "pipemax_xfer_get_stats": (C.c_int, [C.c_void_p, C.POINTER(XferStats)]),
    "pipemax_xfer_reset_stats": (C.c_int, [C.c_void_p]),
    "pipemax_xfer_get_log": (C.c_int, [C.c_void_p, C.POINTER(XferLog), C.c_int]),
    "pipemax_xfer_debug_set_host_us_per_mib": (C.c_int, [C.c_void_p, C.c_int]),
    "pipemax_xfer_debug_pause": (C.c_int, [C.c_void_p, C.c_int]),
    "pipemax_stage_attach_xfer": (C.c_int, [C.c_void_p, C.c_void_p]),
    "pipemax_sched_create": (C.c_int, [C.POINTER(SchedConfig), C.POINTER(C.c_void_p)]),
    "pipemax_sched_destroy": (C.c_int, [C.c_void_p]),
    "pipemax_sched_predict": (C.c_double, [C.c_void_p, C.c_int32, C.c_int64]),
    "pipemax_sched_budget": (C.c_int64, [C.c_void_p, C.c_double]),
    "pipemax_sched_observe": (C.c_int, [C.c_void_p, C.c_int64]),
    "pipemax_sched_short_first_fill": (C.c_int, [_i32p, C.c_int32, C.c_int64, _i32p, _i32p]),
    "pipemax_sched_greedy_fill": (C.c_int, [_i32p, C.c_int32, C.c_int64, _i32p, _i32p]),
    "pipemax_sched_refine": (C.c_int, [C.c_void_p, _i32p, C.c_int32, C.c_int64, C.c_double, _i32p, _i32p, _i32p]),
    "pipemax_sched_partition": (C.c_int, [_i32p, C.c_int32, C.c_int32, _i32p]),
    "pipemax_sched_set_batch": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, _i32p, _i32p]),
    "pipemax_sched_set_gpu_pages_free": (C.c_int, [C.c_void_p, C.c_int64]),
    "pipemax_sched_attach": (C.c_int, [C.c_void_p, C.c_void_p]),
    "pipemax_sched_plan": (C.c_int, [C.c_void_p, C.c_int64, C.POINTER(SchedIter), _i32p, _i32p, _i32p]),
    "pipemax_sched_iterate": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(SchedIter), _i32p, _i32p, _i32p]),
    "pipemax_get_config": (C.c_int, [C.c_void_p, C.POINTER(Config)]),
    "pipemax_mb_size": (C.c_int, [C.c_void_p, C.c_int, _i32p]),
    "pipemax_stage_create": (C.c_int, [C.POINTER(Config), C.POINTER(_vp)]),
    "pipemax_stage_destroy": (C.c_int, [_vp]),
    "pipemax_set_weight": (C.c_int, [_vp, C.c_int, C.c_int, _vp, C.c_size_t]),
    "pipemax_mb_define": (C.c_int, [_vp, C.c_int, C.c_int, _i32p]),
    "pipemax_mb_define_alias": (C.c_int, [_vp, C.c_int, C.c_int]),
    "pipemax_mb_alias_of": (C.c_int, [_vp, C.c_int, _i32p]),
    "pipemax_kv_host_write": (C.c_int, [_vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp]),
    "pipemax_kv_host_read": (C.c_int, [_vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp]),
    "pipemax_kv_dev_read": (C.c_int, [_vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp]),
    "pipemax_prefetch_kv": (C.c_int, [_vp, C.c_int, _i32p, C.c_int]),
    "pipemax_decode_step": (C.c_int, [_vp, C.c_int, _vp, _vp, _vp]),
    "pipemax_decode_step_noalloc": (C.c_int, [_vp, C.c_int, _vp, _vp, _vp]),
    "pipemax_decode_step_seqs": (C.c_int, [_vp, C.c_int, _i32p, C.c_int, _vp, _vp, _vp]),
    "pipemax_prefill": (C.c_int, [_vp, C.c_int, C.c_int, C.c_int, _vp, _vp, _vp]),
    "pipemax_evict_kv": (C.c_int, [_vp, C.c_int, _i32p, C.c_int]),
    "pipemax_sync": (C.c_int, [_vp]),
    "pipemax_get_stats": (C.c_int, [_vp, C.POINTER(Stats)]),
    "pipemax_reset_stats": (C.c_int, [_vp]),
    "pipemax_set_flags": (C.c_int, [_vp, C.c_uint32, C.c_uint32]),
    "pipemax_probe_copy": (C.c_int, [_vp, _vp, C.c_size_t, _vp]),
    "pipemax_probe_read": (C.c_int, [_vp, C.c_size_t, C.c_int, _vp, _vp]),
    "pipemax_probe_link": (C.c_int, [C.c_int, C.c_size_t, C.c_size_t, C.c_size_t, C.c_int, C.c_int,
                                     C.POINTER(LinkProbe)]),
    "pipemax_probe_launch": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(LaunchProbe)]),
    "pipemax_probe_link_strided": (C.c_int, [C.c_int, C.c_size_t, C.c_size_t, C.c_int, C.c_int, C.c_int,
                                        C.POINTER(LinkProbe)]),
    "pipemax_get_ctx_lens": (C.c_int, [_vp, C.c_int, _i32p]),
    "pipemax_get_residency": (C.c_int, [_vp, C.c_int, _i32p]),
    "pipemax_get_block_table": (C.c_int, [_vp, C.c_int, C.c_int, _i32p, _i32p, C.POINTER(C.c_int)]),
    "pipemax_get_layer_outputs": (C.c_int, [_vp, _vp, C.c_size_t]),
    "pipemax_debug_fill_free_gpu_pages": (C.c_int, [_vp, C.c_uint16]),
    "pipemax_debug_set_delays": (C.c_int, [_vp, C.c_int, C.c_int, C.c_int]),
    "pipemax_last_error": (C.c_char_p, []),
    "pipemax_version": (C.c_char_p, []),
    "pipemax_page_elem_offset": (C.c_int64, [C.c_int] * 8),
    "pipemax_plan_copy_runs": (C.c_int, [_i32p, _i32p, C.c_int, C.c_int, _i32p]),
    "pipemax_plan_gemm_splits": (C.c_int, [C.c_int, C.c_int, C.c_int, _i32p, _i32p, _i32p]),
    "pipemax_plan_attention_chunks": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int, _i32p, _i32p, _i32p]),
    "pipemax_pool_create": (C.c_int, [C.c_int, C.POINTER(_vp)]),
    "pipemax_pool_destroy": (C.c_int, [_vp]),
    "pipemax_pool_alloc": (C.c_int, [_vp, C.c_int, _i32p]),
    "pipemax_pool_free": (C.c_int, [_vp, _i32p, C.c_int]),
    "pipemax_pool_free_count": (C.c_int, [_vp]),
}
for _name, (_res, _args) in _sig.items():
    _f = getattr(_lib, _name)
    _f.restype, _f.argtypes = _res, _args


class PipemaxError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"pipemax status {code}: {msg}")
        self.code = code


def last_error() -> str:
    return _lib.pipemax_last_error().decode()


def version() -> str:
    return _lib.pipemax_version().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise PipemaxError(rc, last_error())


def _ids(seq_ids):
    if seq_ids is None:
        return None, 0
    a = np.ascontiguousarray(seq_ids, dtype=np.int32)
    return a.ctypes.data_as(_i32p), int(a.size)


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


class Stage:
    """Thin owner of a pipemax_stage_t; method names follow the C entry points."""

    def __init__(self, *, n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, rope_base, rms_eps,
                 dtype, n_microbatches, max_seqs_per_mb, max_ctx, gpu_kv_bytes, host_kv_bytes,
                 device=0, flags=0, page_tokens=16, host_reserve_tokens=0, wb_layers_per_copy=0):
        self.cfg = Config(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, rope_base, rms_eps,
                          dtype, page_tokens, n_microbatches, max_seqs_per_mb, max_ctx,
                          int(gpu_kv_bytes), int(host_kv_bytes), device, flags, host_reserve_tokens,
                          wb_layers_per_copy)
        self._h = _vp()
        _check(_lib.pipemax_stage_create(C.byref(self.cfg), C.byref(self._h)))
        self.np_dtype = np.float32 if dtype == F32 else np.uint16
        self._nseq = {}

    def destroy(self):
        if self._h:
            _check(_lib.pipemax_stage_destroy(self._h))
            self._h = _vp()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- set-up ---------------------------------------------------------------------------
    def set_weight(self, layer: int, which: int, arr: np.ndarray):
        a = np.ascontiguousarray(arr, dtype=self.np_dtype)
        _check(_lib.pipemax_set_weight(self._h, layer, which, _ptr(a), a.nbytes))

    def mb_define(self, mb: int, ctx_lens):
        a = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        _check(_lib.pipemax_mb_define(self._h, mb, int(a.size), a.ctypes.data_as(_i32p)))
        self._nseq[mb] = int(a.size)

    def mb_define_alias(self, mb: int, src_mb: int):
        _check(_lib.pipemax_mb_define_alias(self._h, mb, src_mb))
        self._nseq[mb] = self._nseq[src_mb]

    def mb_alias_of(self, mb: int) -> int:
        out = C.c_int32(0)
        _check(_lib.pipemax_mb_alias_of(self._h, mb, C.byref(out)))
        return int(out.value)

    def kv_host_write(self, mb, seq, layer, tok0, K: np.ndarray, V: np.ndarray):
        K = np.ascontiguousarray(K, dtype=self.np_dtype)
        V = np.ascontiguousarray(V, dtype=self.np_dtype)
        assert K.shape == V.shape
        _check(_lib.pipemax_kv_host_write(self._h, mb, seq, layer, tok0, K.shape[0], _ptr(K), _ptr(V)))

    def _kv_read(self, fn, mb, seq, layer, tok0, ntok):
        shp = (ntok, self.cfg.n_kv_heads, self.cfg.head_dim)
        K = np.empty(shp, dtype=self.np_dtype)
        V = np.empty(shp, dtype=self.np_dtype)
        _check(fn(self._h, mb, seq, layer, tok0, ntok, _ptr(K), _ptr(V)))
        return K, V

    def kv_host_read(self, mb, seq, layer, tok0, ntok):
        return self._kv_read(_lib.pipemax_kv_host_read, mb, seq, layer, tok0, ntok)

    def kv_dev_read(self, mb, seq, layer, tok0, ntok):
        return self._kv_read(_lib.pipemax_kv_dev_read, mb, seq, layer, tok0, ntok)

    # -- hot path -------------------------------------------------------------------------
    def prefetch_kv(self, mb, seq_ids=None):
        p, n = _ids(seq_ids)
        _check(_lib.pipemax_prefetch_kv(self._h, mb, p, n))

    def decode_step(self, mb, hidden_in_ptr: int, hidden_out_ptr: int, stream_ptr: int = 0):
        """Device pointers as integers (e.g. tensor.data_ptr(), torch stream .cuda_stream)."""
        _check(_lib.pipemax_decode_step(self._h, mb, _vp(hidden_in_ptr), _vp(hidden_out_ptr),
                                        _vp(stream_ptr) if stream_ptr else None))

    def decode_step_noalloc(self, mb, hidden_in_ptr: int, hidden_out_ptr: int, stream_ptr: int = 0):
        """pipemax_decode_step with the working buffers in the library's static per-GPU scratch."""
        _check(_lib.pipemax_decode_step_noalloc(self._h, mb, _vp(hidden_in_ptr), _vp(hidden_out_ptr),
                                                _vp(stream_ptr) if stream_ptr else None))

    def decode_step_seqs(self, mb, seq_ids, hidden_in_ptr: int, hidden_out_ptr: int, stream_ptr: int = 0):
        """Rows of the hidden tensors follow seq_ids (distinct sequence indices of mb)."""
        a = np.ascontiguousarray(seq_ids, dtype=np.int32)
        _check(_lib.pipemax_decode_step_seqs(self._h, mb, a.ctypes.data_as(_i32p), int(a.size),
                                             _vp(hidden_in_ptr), _vp(hidden_out_ptr),
                                             _vp(stream_ptr) if stream_ptr else None))

    def prefill(self, mb, seq, n_tokens, hidden_in_ptr: int, hidden_out_ptr: int, stream_ptr: int = 0):
        """n_tokens new tokens of one sequence; hidden tensors are [n_tokens][hidden] on the device."""
        _check(_lib.pipemax_prefill(self._h, mb, seq, n_tokens, _vp(hidden_in_ptr), _vp(hidden_out_ptr),
                                    _vp(stream_ptr) if stream_ptr else None))

    def attach_xfer(self, xfer):
        """Prefetch copies go through a transfer orchestrator (None detaches)."""
        _check(_lib.pipemax_stage_attach_xfer(self._h, xfer._h if xfer is not None else None))
        self._xfer = xfer           # keeps it alive

    def evict_kv(self, mb, seq_ids=None):
        p, n = _ids(seq_ids)
        _check(_lib.pipemax_evict_kv(self._h, mb, p, n))

    def sync(self):
        _check(_lib.pipemax_sync(self._h))

    # -- introspection --------------------------------------------------------------------
    def get_stats(self) -> dict:
        s = Stats()
        _check(_lib.pipemax_get_stats(self._h, C.byref(s)))
        return s.as_dict()

    def reset_stats(self):
        _check(_lib.pipemax_reset_stats(self._h))

    def set_flags(self, set_: int = 0, clear: int = 0):
        _check(_lib.pipemax_set_flags(self._h, set_, clear))

    def get_ctx_lens(self, mb) -> np.ndarray:
        out = np.empty(self._nseq[mb], dtype=np.int32)
        _check(_lib.pipemax_get_ctx_lens(self._h, mb, out.ctypes.data_as(_i32p)))
        return out

    def get_residency(self, mb) -> np.ndarray:
        out = np.empty(self._nseq[mb], dtype=np.int32)
        _check(_lib.pipemax_get_residency(self._h, mb, out.ctypes.data_as(_i32p)))
        return out

    def get_block_table(self, mb, seq):
        n = C.c_int(0)
        _check(_lib.pipemax_get_block_table(self._h, mb, seq, None, None, C.byref(n)))
        g = np.empty(max(n.value, 1), dtype=np.int32)
        h = np.empty(max(n.value, 1), dtype=np.int32)
        m = C.c_int(n.value)
        _check(_lib.pipemax_get_block_table(self._h, mb, seq, g.ctypes.data_as(_i32p),
                                            h.ctypes.data_as(_i32p), C.byref(m)))
        return g[: m.value], h[: m.value]

    def debug_fill_free_gpu_pages(self, pattern: int):
        _check(_lib.pipemax_debug_fill_free_gpu_pages(self._h, pattern))

    def debug_set_delays(self, h2d_us: int = 0, d2h_us: int = 0, worker_us: int = 0):
        _check(_lib.pipemax_debug_set_delays(self._h, h2d_us, d2h_us, worker_us))

    def get_layer_outputs(self, b: int) -> np.ndarray:
        out = np.empty((self.cfg.n_layers, b, self.cfg.hidden), dtype=np.float32)
        _check(_lib.pipemax_get_layer_outputs(self._h, _ptr(out), out.nbytes))
        return out


def probe_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream_ptr: int = 0):
    _check(_lib.pipemax_probe_copy(_vp(dst_ptr), _vp(src_ptr), nbytes, _vp(stream_ptr) if stream_ptr else None))


# -- host-side planning helpers ---------------------------------------------------------------
def probe_read(src_ptr: int, nbytes: int, segment_trips: int, sink_ptr: int, stream_ptr: int = 0):
    _check(_lib.pipemax_probe_read(_vp(src_ptr), nbytes, segment_trips, _vp(sink_ptr),
                                   _vp(stream_ptr) if stream_ptr else None))


def probe_link(total_bytes: int, piece_bytes: int, piece_stride: int | None = None, direction: int = 0,
               repeats: int = 3, device: int = 0) -> dict:
    out = LinkProbe()
    _check(_lib.pipemax_probe_link(device, total_bytes, piece_bytes, piece_stride or piece_bytes, direction, repeats,
                                   C.byref(out)))
    return {k: getattr(out, k) for k, _ in LinkProbe._fields_}


def probe_launch(n_kernels: int, use_graph: bool, repeats: int = 20, device: int = 0) -> dict:
    out = LaunchProbe()
    _check(_lib.pipemax_probe_launch(device, n_kernels, int(use_graph), repeats, C.byref(out)))
    return {k: getattr(out, k) for k, _ in LaunchProbe._fields_}


def probe_link_2d(row_bytes: int, host_pitch: int, rows_per_copy: int, n_copies: int, repeats: int = 3,
                  device: int = 0) -> dict:
    out = LinkProbe()
    _check(_lib.pipemax_probe_link_strided(device, row_bytes, host_pitch, rows_per_copy, n_copies, repeats, C.byref(out)))
    return {k: getattr(out, k) for k, _ in LinkProbe._fields_}


def page_elem_offset(n_layers, n_kv_heads, head_dim, layer, kv, head, tok, dd) -> int:
    return int(_lib.pipemax_page_elem_offset(n_layers, n_kv_heads, head_dim, layer, kv, head, tok, dd))


def plan_copy_runs(src_pages, dst_pages, max_run_pages: int):
    s = np.ascontiguousarray(src_pages, dtype=np.int32)
    d = np.ascontiguousarray(dst_pages, dtype=np.int32)
    assert s.size == d.size
    runs = np.empty(3 * max(int(s.size), 1), dtype=np.int32)
    n = _lib.pipemax_plan_copy_runs(s.ctypes.data_as(_i32p), d.ctypes.data_as(_i32p), int(s.size),
                                    max_run_pages, runs.ctypes.data_as(_i32p))
    if n < 0:
        raise PipemaxError(n, last_error())
    return runs[: 3 * n].reshape(n, 3)


def plan_attention_chunks(n_seqs: int, n_kv_heads: int, max_ctx_tokens: int, sum_pages: int, compute_units: int = 256):
    """(pages per item, chunks of the longest sequence, whether a wave (True) or a work-group streams an item) the
    stage plans for such a step on a GPU of that many compute units."""
    cp, nch, pw = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(_lib.pipemax_plan_attention_chunks(n_seqs, n_kv_heads, max_ctx_tokens, sum_pages, compute_units,
                                              C.byref(cp), C.byref(nch), C.byref(pw)))
    return int(cp.value), int(nch.value), bool(pw.value)


def plan_gemm_splits(rows: int, n_cols: int, k: int):
    """(planned splits, splits of the launch geometry, k-steps per split) of the large-tile GEMM."""
    out = (C.c_int32 * 3)()
    _check(_lib.pipemax_plan_gemm_splits(rows, n_cols, k, C.cast(C.byref(out, 0), _i32p),
                                         C.cast(C.byref(out, 4), _i32p), C.cast(C.byref(out, 8), _i32p)))
    return int(out[0]), int(out[1]), int(out[2])


class Pool:
    def __init__(self, n_pages: int):
        self._h = _vp()
        _check(_lib.pipemax_pool_create(n_pages, C.byref(self._h)))

    def alloc(self, n: int) -> np.ndarray:
        out = np.empty(max(n, 1), dtype=np.int32)
        _check(_lib.pipemax_pool_alloc(self._h, n, out.ctypes.data_as(_i32p)))
        return out[:n]

    def free(self, pages):
        a = np.ascontiguousarray(pages, dtype=np.int32)
        _check(_lib.pipemax_pool_free(self._h, a.ctypes.data_as(_i32p), int(a.size)))

    def free_count(self) -> int:
        return int(_lib.pipemax_pool_free_count(self._h))

    def __del__(self):
        if self._h:
            _lib.pipemax_pool_destroy(self._h)
            self._h = _vp()


# -- prefetch-aware decode scheduler (include/pipemax_sched.h) ------------------------------------
def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


def sched_short_first_fill(lens, budget: int) -> list:
    a, p = _i32(lens)
    sel, n = np.empty(max(a.size, 1), dtype=np.int32), C.c_int32(0)
    _check(_lib.pipemax_sched_short_first_fill(p, int(a.size), int(budget), sel.ctypes.data_as(_i32p), C.byref(n)))
    return sel[: n.value].tolist()


def sched_greedy_fill(lens, budget: int) -> list:
    a, p = _i32(lens)
    sel, n = np.empty(max(a.size, 1), dtype=np.int32), C.c_int32(0)
    _check(_lib.pipemax_sched_greedy_fill(p, int(a.size), int(budget), sel.ctypes.data_as(_i32p), C.byref(n)))
    return sel[: n.value].tolist()


def sched_partition(lens, n_batches: int) -> list:
    a, p = _i32(lens)
    out = np.empty(max(a.size, 1), dtype=np.int32)
    _check(_lib.pipemax_sched_partition(p, int(a.size), n_batches, out.ctypes.data_as(_i32p)))
    return out[: a.size].tolist()


class Scheduler:
    """Thin wrapper of pipemax_sched_t (argument marshalling only)."""

    def __init__(self, *, alpha_s, beta_s, delta_s, link_tokens_per_s, n_batches, window=8, steady_rel_range=0.05,
                 max_refine_steps=16, refine_tol_s=None, static_budget_tokens=0, page_tokens=16):
        self.cfg = SchedConfig(alpha_s=alpha_s, beta_s=beta_s, delta_s=delta_s, link_tokens_per_s=link_tokens_per_s,
                               steady_rel_range=steady_rel_range,
                               refine_tol_s=alpha_s / 2 if refine_tol_s is None else refine_tol_s,
                               static_budget_tokens=static_budget_tokens, window=window,
                               max_refine_steps=max_refine_steps, n_batches=n_batches, page_tokens=page_tokens)
        self._h = _vp()
        self._cap = 1
        _check(_lib.pipemax_sched_create(C.byref(self.cfg), C.byref(self._h)))

    def destroy(self):
        if self._h:
            _check(_lib.pipemax_sched_destroy(self._h))
            self._h = _vp()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def predict(self, b: int, total_len: int) -> float:
        return float(_lib.pipemax_sched_predict(self._h, int(b), int(total_len)))

    def budget(self, t_hat_s: float) -> int:
        return int(_lib.pipemax_sched_budget(self._h, float(t_hat_s)))

    def observe(self, budget_tokens: int) -> bool:
        rc = _lib.pipemax_sched_observe(self._h, int(budget_tokens))
        _check(min(rc, 0))
        return bool(rc)

    def refine(self, lens, budget: int, gap_s: float, sel):
        a, p = _i32(lens)
        buf = np.empty(max(a.size, 1), dtype=np.int32)
        buf[: len(sel)] = sel
        n, ex = C.c_int32(len(sel)), C.c_int32(0)
        _check(_lib.pipemax_sched_refine(self._h, p, int(a.size), int(budget), float(gap_s),
                                         buf.ctypes.data_as(_i32p), C.byref(n), C.byref(ex)))
        return buf[: n.value].tolist(), ex.value

    def set_batch(self, mb: int, lens, resident):
        a, p = _i32(lens)
        r, q = _i32(resident)
        assert a.size == r.size
        _check(_lib.pipemax_sched_set_batch(self._h, mb, int(a.size), p, q))
        self._cap = max(self._cap, int(a.size))

    def set_gpu_pages_free(self, pages: int):
        _check(_lib.pipemax_sched_set_gpu_pages_free(self._h, int(pages)))

    def attach(self, stage: "Stage"):
        _check(_lib.pipemax_sched_attach(self._h, stage._h))
        self._cap = max(self._cap, int(stage.cfg.max_seqs_per_mb))

    def _result(self, it, e, p, v):
        d = {n: getattr(it, n) for n, _ in it._fields_}
        d["exec"] = e[: it.n_exec].tolist()
        d["prefetch"] = p[: it.n_prefetch].tolist()
        d["evict"] = v[: it.n_evict].tolist()
        return d

    def plan(self, t: int) -> dict:
        it = SchedIter()
        e, p, v = (np.empty(self._cap, dtype=np.int32) for _ in range(3))
        _check(_lib.pipemax_sched_plan(self._h, int(t), C.byref(it), e.ctypes.data_as(_i32p),
                                       p.ctypes.data_as(_i32p), v.ctypes.data_as(_i32p)))
        return self._result(it, e, p, v)

    def iterate(self, stage: "Stage", t: int, hidden_in_ptr: int, hidden_out_ptr: int, stream_ptr: int = 0) -> dict:
        it = SchedIter()
        e, p, v = (np.empty(self._cap, dtype=np.int32) for _ in range(3))
        _check(_lib.pipemax_sched_iterate(self._h, stage._h, int(t), _vp(hidden_in_ptr), _vp(hidden_out_ptr),
                                          _vp(stream_ptr) if stream_ptr else None, C.byref(it),
                                          e.ctypes.data_as(_i32p), p.ctypes.data_as(_i32p), v.ctypes.data_as(_i32p)))
        return self._result(it, e, p, v)


# -- demand-priority transfer orchestrator (include/pipemax_xfer.h) ---------------------------------
class Xfer:
    """Thin wrapper of pipemax_xfer_t.  Pointers are integers (tensor.data_ptr(), ndarray.ctypes.data)."""

    def __init__(self, device: int = 0, max_inflight_bulk: int = 2, chunk_bytes: int = 4 << 20, log_capacity: int = 0):
        self.cfg = XferConfig(device=device, max_inflight_bulk=max_inflight_bulk, chunk_bytes=chunk_bytes,
                              log_capacity=log_capacity)
        self._h = _vp()
        _check(_lib.pipemax_xfer_create(C.byref(self.cfg), C.byref(self._h)))

    def destroy(self):
        if self._h:
            _check(_lib.pipemax_xfer_destroy(self._h))
            self._h = _vp()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def submit(self, kind: int, direction: int, dst_ptr: int, src_ptr: int, nbytes: int) -> int:
        t = C.c_uint64(0)
        _check(_lib.pipemax_xfer_submit(self._h, kind, direction, _vp(dst_ptr), _vp(src_ptr), nbytes, C.byref(t)))
        return t.value

    def wait(self, ticket: int):
        _check(_lib.pipemax_xfer_wait(self._h, ticket))

    def poll(self, ticket: int) -> bool:
        rc = _lib.pipemax_xfer_poll(self._h, ticket)
        _check(min(rc, 0))
        return bool(rc)

    def stream_wait(self, ticket: int, stream_ptr: int):
        _check(_lib.pipemax_xfer_stream_wait(self._h, ticket, _vp(stream_ptr)))

    def drain(self):
        _check(_lib.pipemax_xfer_drain(self._h))

    def stats(self) -> dict:
        s = XferStats()
        _check(_lib.pipemax_xfer_get_stats(self._h, C.byref(s)))
        return {k: {"urgent": getattr(s, k)[0], "bulk": getattr(s, k)[1]} for k, _ in s._fields_}

    def reset_stats(self):
        _check(_lib.pipemax_xfer_reset_stats(self._h))

    def log(self, capacity: int = 4096) -> list:
        buf = (XferLog * capacity)()
        n = _lib.pipemax_xfer_get_log(self._h, buf, capacity)
        _check(min(n, 0))
        return [(e.ticket, e.offset, e.bytes, e.kind, e.dir) for e in buf[:n]]

    def debug_pause(self, paused: bool):
        _check(_lib.pipemax_xfer_debug_pause(self._h, int(paused)))

    def debug_set_host_us_per_mib(self, us: int):
        _check(_lib.pipemax_xfer_debug_set_host_us_per_mib(self._h, us))
