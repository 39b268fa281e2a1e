"""ctypes binding of libefim: argument marshalling only.

Every function has the name and argument order of its C counterpart in
``include/efim.h``.  Device buffers are passed as torch tensors (or raw
integer addresses); nothing is computed here and there is no fallback: if the
HIP library cannot be loaded the import fails.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

EFIM_OK = 0
EFIM_ERR_INVALID_ARG = -1
EFIM_ERR_UNSUPPORTED = -2
EFIM_ERR_WORKSPACE = -3
EFIM_ERR_LAUNCH = -4

EFIM_TUNE_SPLIT_KV = 0
EFIM_TUNE_XCD_GROUPING = 1
EFIM_TUNE_NUM_SLOTS = 2
EFIM_TUNE_ROW_TILE = 3
EFIM_TUNE_FUSED_MERGE = 4
EFIM_TUNE_DEVICE_PLAN = 5


class EfimBatch(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
        ("max_pages_per_req", ctypes.c_int32),
        ("num_pages", ctypes.c_int64),
        ("cached_len", ctypes.c_void_p),
        ("new_len", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p),
    ]


class EfimWorkItem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "req", "kv_head", "row_begin", "row_count", "key_begin", "key_end", "partial_slot", "merge_id")]


WORK_ITEM_DTYPE = np.dtype([(n, np.int32) for n, _ in EfimWorkItem._fields_])


class EfimError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = _lib.efim_status_string(status).decode()
        if status == EFIM_ERR_LAUNCH:
            msg += " (hipError %d)" % _lib.efim_last_hip_error()
        super().__init__("%s: %s" % (where, msg))


class EfimPromptInfo(ctypes.Structure):
    """efim_prompt_info_t"""
    _fields_ = [("order", ctypes.c_int32), ("reserved", ctypes.c_int32), ("common_len", ctypes.c_int64),
                ("inc_len", ctypes.c_int64), ("suffix_len", ctypes.c_int64), ("prompt_len", ctypes.c_int64),
                ("cached_len", ctypes.c_int64), ("new_len", ctypes.c_int64)]


def _load():
    path = os.environ.get("EFIM_LIBRARY")  # explicit path to an already built libefim.so
    if not path:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            _build.build_library()
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    bp = ctypes.POINTER(EfimBatch)
    lib.efim_rope_append.argtypes = [bp, vp, vp, vp, vp, vp, ctypes.c_double, i32, vp]
    lib.efim_rope_append.restype = i32
    lib.efim_rope_append_table.argtypes = [bp, vp, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_double), i32, i32, vp]
    lib.efim_rope_append_table.restype = i32
    lib.efim_extend_workspace_bytes.argtypes = [bp]
    lib.efim_extend_workspace_bytes.restype = ctypes.c_size_t
    lib.efim_extend_attention.argtypes = [bp, vp, vp, vp, vp, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.efim_extend_attention.restype = i32
    lib.efim_extend_static_limit_bytes.argtypes = []
    lib.efim_extend_static_limit_bytes.restype = ctypes.c_size_t
    lib.efim_extend_attention_static.argtypes = [bp, vp, vp, vp, vp, ctypes.c_float, vp]
    lib.efim_extend_attention_static.restype = i32
    lib.efim_plan_create.argtypes = [bp, i32]
    lib.efim_plan_create.restype = vp
    lib.efim_plan_destroy.argtypes = [vp]
    lib.efim_plan_destroy.restype = None
    lib.efim_plan_workspace_bytes.argtypes = [vp]
    lib.efim_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.efim_plan_upload.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.efim_plan_upload.restype = i32
    lib.efim_extend_attention_planned.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.efim_extend_attention_planned.restype = i32
    lib.efim_decode_step_planned.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_double, i32, ctypes.c_float, vp, vp]
    lib.efim_decode_step_planned.restype = i32
    lib.efim_stream_release.argtypes = [vp]
    lib.efim_stream_release.restype = i32
    lib.efim_source_digest.argtypes = []
    lib.efim_source_digest.restype = ctypes.c_char_p
    lib.efim_decode_workspace_bytes.argtypes = [bp]
    lib.efim_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.efim_decode_step.argtypes = [bp, vp, vp, vp, vp, vp, vp, ctypes.c_double, i32, ctypes.c_float, vp,
                                     ctypes.c_size_t, vp]
    lib.efim_decode_step.restype = i32
    lib.efim_decode_step_table.argtypes = [bp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_double), i32, i32,
                                           ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.efim_decode_step_table.restype = i32
    f32 = ctypes.c_float
    lib.efim_rope_append_fp8.argtypes = [bp, vp, vp, vp, vp, vp, ctypes.c_double, i32, f32, f32, vp]
    lib.efim_rope_append_fp8.restype = i32
    lib.efim_extend_attention_fp8.argtypes = [bp, vp, vp, vp, vp, f32, f32, f32, vp, ctypes.c_size_t, vp]
    lib.efim_extend_attention_fp8.restype = i32
    lib.efim_decode_step_fp8.argtypes = [bp, vp, vp, vp, vp, vp, vp, ctypes.c_double, i32, f32, f32, f32, vp,
                                         ctypes.c_size_t, vp]
    lib.efim_decode_step_fp8.restype = i32
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.efim_rope_append_fp8_table.argtypes = [bp, vp, vp, vp, vp, vp, f64p, i32, i32, f32, f32, vp]
    lib.efim_rope_append_fp8_table.restype = i32
    lib.efim_decode_step_fp8_table.argtypes = [bp, vp, vp, vp, vp, vp, vp, f64p, i32, i32, f32, f32, f32, vp,
                                               ctypes.c_size_t, vp]
    lib.efim_decode_step_fp8_table.restype = i32
    lib.efim_extend_plan_items.argtypes = [bp, vp, i64]
    lib.efim_extend_plan_items.restype = i64
    lib.efim_set_tuning.argtypes = [i32, i32]
    lib.efim_set_tuning.restype = i32
    lib.efim_set_kernel_events.argtypes = [vp, vp]
    lib.efim_set_kernel_events.restype = i32
    lib.efim_status_string.argtypes = [i32]
    lib.efim_status_string.restype = ctypes.c_char_p
    lib.efim_last_hip_error.argtypes = []
    lib.efim_last_hip_error.restype = i32
    lib.efim_version.argtypes = []
    lib.efim_version.restype = i32
    ip = ctypes.POINTER(ctypes.c_int32)
    lib.efim_session_pool_create.argtypes = [i32, i32, i32, i32, i32]
    lib.efim_session_pool_create.restype = vp
    lib.efim_session_pool_destroy.argtypes = [vp]
    lib.efim_session_pool_destroy.restype = None
    lib.efim_session_transform.argtypes = [vp, ctypes.c_uint64, ip, i64, ip, i64, ctypes.POINTER(EfimPromptInfo)]
    lib.efim_session_transform.restype = i32
    lib.efim_session_prompt.argtypes = [vp, ctypes.c_uint64, ip, i64]
    lib.efim_session_prompt.restype = i64
    lib.efim_session_drop.argtypes = [vp, ctypes.c_uint64]
    lib.efim_session_drop.restype = i32
    lib.efim_session_count.argtypes = [vp]
    lib.efim_session_count.restype = i64
    return lib


_lib = _load()
LIBRARY_PATH = os.environ.get("EFIM_LIBRARY") or _build.LIB_PATH
EXPORTED_SYMBOLS = (
    "efim_rope_append", "efim_rope_append_table", "efim_extend_workspace_bytes", "efim_extend_attention",
    "efim_extend_static_limit_bytes", "efim_extend_attention_static",
    "efim_decode_workspace_bytes", "efim_decode_step", "efim_decode_step_table",
    "efim_rope_append_fp8", "efim_extend_attention_fp8", "efim_decode_step_fp8",
    "efim_rope_append_fp8_table", "efim_decode_step_fp8_table",
    "efim_extend_plan_items", "efim_set_tuning", "efim_set_kernel_events", "efim_status_string",
    "efim_last_hip_error", "efim_version", "efim_source_digest", "efim_stream_release",
    "efim_plan_create", "efim_plan_destroy", "efim_plan_workspace_bytes", "efim_plan_upload",
    "efim_extend_attention_planned", "efim_decode_step_planned",
    "efim_session_pool_create", "efim_session_pool_destroy", "efim_session_transform", "efim_session_prompt",
    "efim_session_drop", "efim_session_count",
)


def _ptr(x):
    """Address of a torch tensor / numpy array, or an integer address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError("cannot take the address of %r" % type(x))


def _stream_ptr(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class BatchDesc:
    """Owns the host arrays behind an efim_batch_t and keeps the device block table alive."""

    def __init__(self, cached_len, new_len, block_table, num_q_heads, num_kv_heads, head_dim,
                 page_size, num_pages, max_pages_per_req=None):
        self.cached_len = np.ascontiguousarray(cached_len, dtype=np.int32)
        self.new_len = np.ascontiguousarray(new_len, dtype=np.int32)
        self.block_table = block_table
        if max_pages_per_req is None:
            max_pages_per_req = int(block_table.shape[1]) if hasattr(block_table, "shape") else 0
        self.c = EfimBatch(
            int(self.cached_len.shape[0]), num_q_heads, num_kv_heads, head_dim, page_size,
            max_pages_per_req, num_pages,
            self.cached_len.ctypes.data if self.cached_len.size else None,
            self.new_len.ctypes.data if self.new_len.size else None,
            _ptr(block_table))

    @property
    def total_new(self):
        return int(self.new_len.sum())


def _check(status, where):
    if status != EFIM_OK:
        raise EfimError(status, where)


def efim_rope_append(batch, q, k_new, v_new, k_cache, v_cache, rope_base, rope_interleaved=0, stream=None):
    _check(_lib.efim_rope_append(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                 _ptr(v_cache), float(rope_base), int(rope_interleaved), _stream_ptr(stream)),
           "efim_rope_append")


def efim_rope_append_table(batch, q, k_new, v_new, k_cache, v_cache, inv_freq, rotary_dim, rope_interleaved=0,
                           stream=None):
    table = np.ascontiguousarray(np.asarray(inv_freq, dtype=np.float64).reshape(-1))
    assert table.size >= int(rotary_dim) // 2, "inv_freq needs rotary_dim / 2 entries"
    _check(_lib.efim_rope_append_table(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                       _ptr(v_cache), table.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                       int(rotary_dim), int(rope_interleaved), _stream_ptr(stream)),
           "efim_rope_append_table")


def efim_extend_workspace_bytes(batch):
    return int(_lib.efim_extend_workspace_bytes(ctypes.byref(batch.c)))


def efim_extend_attention(batch, q, k_cache, v_cache, out, sm_scale, workspace, workspace_bytes, stream=None):
    _check(_lib.efim_extend_attention(ctypes.byref(batch.c), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out),
                                      float(sm_scale), _ptr(workspace), int(workspace_bytes), _stream_ptr(stream)),
           "efim_extend_attention")


def efim_extend_static_limit_bytes():
    return int(_lib.efim_extend_static_limit_bytes())


def efim_extend_attention_static(batch, q, k_cache, v_cache, out, sm_scale, stream=None):
    _check(_lib.efim_extend_attention_static(ctypes.byref(batch.c), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                             _ptr(out), float(sm_scale), _stream_ptr(stream)),
           "efim_extend_attention_static")


class Plan:
    """efim_plan_t: owns the handle; close() (or garbage collection) destroys it."""

    def __init__(self, batch, decode=False):
        self.handle = _lib.efim_plan_create(ctypes.byref(batch.c), 1 if decode else 0)
        if not self.handle:
            raise EfimError(EFIM_ERR_INVALID_ARG, "efim_plan_create")

    def close(self):
        if getattr(self, "handle", None):
            _lib.efim_plan_destroy(self.handle)
            self.handle = None

    __del__ = close


def efim_plan_workspace_bytes(plan):
    return int(_lib.efim_plan_workspace_bytes(plan.handle))


def efim_plan_upload(plan, workspace, workspace_bytes, stream=None):
    _check(_lib.efim_plan_upload(plan.handle, _ptr(workspace), int(workspace_bytes), _stream_ptr(stream)),
           "efim_plan_upload")


def efim_extend_attention_planned(plan, block_table, q, k_cache, v_cache, out, sm_scale, workspace, stream=None):
    _check(_lib.efim_extend_attention_planned(plan.handle, _ptr(block_table), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                              _ptr(out), float(sm_scale), _ptr(workspace), _stream_ptr(stream)),
           "efim_extend_attention_planned")


def efim_decode_step_planned(plan, block_table, q, k_new, v_new, k_cache, v_cache, out, rope_base, rope_interleaved,
                             sm_scale, workspace, stream=None):
    _check(_lib.efim_decode_step_planned(plan.handle, _ptr(block_table), _ptr(q), _ptr(k_new), _ptr(v_new),
                                         _ptr(k_cache), _ptr(v_cache), _ptr(out), float(rope_base),
                                         int(rope_interleaved), float(sm_scale), _ptr(workspace),
                                         _stream_ptr(stream)),
           "efim_decode_step_planned")


def efim_stream_release(stream=None):
    _check(_lib.efim_stream_release(_stream_ptr(stream)), "efim_stream_release")


def efim_source_digest():
    """Digest of the library's sources as recorded when it was built (see build.source_digest)."""
    return _lib.efim_source_digest().decode()


def efim_decode_workspace_bytes(batch):
    return int(_lib.efim_decode_workspace_bytes(ctypes.byref(batch.c)))


def efim_decode_step(batch, q, k_new, v_new, k_cache, v_cache, out, rope_base, rope_interleaved, sm_scale,
                     workspace, workspace_bytes, stream=None):
    _check(_lib.efim_decode_step(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                 _ptr(v_cache), _ptr(out), float(rope_base), int(rope_interleaved), float(sm_scale),
                                 _ptr(workspace), int(workspace_bytes), _stream_ptr(stream)),
           "efim_decode_step")


def efim_decode_step_table(batch, q, k_new, v_new, k_cache, v_cache, out, inv_freq, rotary_dim, rope_interleaved,
                           sm_scale, workspace, workspace_bytes, stream=None):
    table = np.ascontiguousarray(np.asarray(inv_freq, dtype=np.float64).reshape(-1))
    assert table.size >= int(rotary_dim) // 2, "inv_freq needs rotary_dim / 2 entries"
    _check(_lib.efim_decode_step_table(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                       _ptr(v_cache), _ptr(out), table.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                       int(rotary_dim), int(rope_interleaved), float(sm_scale), _ptr(workspace),
                                       int(workspace_bytes), _stream_ptr(stream)),
           "efim_decode_step_table")


def efim_rope_append_fp8(batch, q, k_new, v_new, k_cache, v_cache, rope_base, rope_interleaved, k_scale, v_scale,
                         stream=None):
    _check(_lib.efim_rope_append_fp8(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                     _ptr(v_cache), float(rope_base), int(rope_interleaved), float(k_scale),
                                     float(v_scale), _stream_ptr(stream)),
           "efim_rope_append_fp8")


def efim_extend_attention_fp8(batch, q, k_cache, v_cache, out, sm_scale, k_scale, v_scale, workspace,
                              workspace_bytes, stream=None):
    _check(_lib.efim_extend_attention_fp8(ctypes.byref(batch.c), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out),
                                          float(sm_scale), float(k_scale), float(v_scale), _ptr(workspace),
                                          int(workspace_bytes), _stream_ptr(stream)),
           "efim_extend_attention_fp8")


def efim_decode_step_fp8(batch, q, k_new, v_new, k_cache, v_cache, out, rope_base, rope_interleaved, sm_scale,
                         k_scale, v_scale, workspace, workspace_bytes, stream=None):
    _check(_lib.efim_decode_step_fp8(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                     _ptr(v_cache), _ptr(out), float(rope_base), int(rope_interleaved),
                                     float(sm_scale), float(k_scale), float(v_scale), _ptr(workspace),
                                     int(workspace_bytes), _stream_ptr(stream)),
           "efim_decode_step_fp8")


def _freq_table(inv_freq, rotary_dim):
    table = np.ascontiguousarray(np.asarray(inv_freq, dtype=np.float64).reshape(-1))
    assert table.size >= int(rotary_dim) // 2, "inv_freq needs rotary_dim / 2 entries"
    return table


def efim_rope_append_fp8_table(batch, q, k_new, v_new, k_cache, v_cache, inv_freq, rotary_dim, rope_interleaved,
                               k_scale, v_scale, stream=None):
    table = _freq_table(inv_freq, rotary_dim)
    _check(_lib.efim_rope_append_fp8_table(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new),
                                           _ptr(k_cache), _ptr(v_cache),
                                           table.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), int(rotary_dim),
                                           int(rope_interleaved), float(k_scale), float(v_scale),
                                           _stream_ptr(stream)),
           "efim_rope_append_fp8_table")


def efim_decode_step_fp8_table(batch, q, k_new, v_new, k_cache, v_cache, out, inv_freq, rotary_dim,
                               rope_interleaved, sm_scale, k_scale, v_scale, workspace, workspace_bytes,
                               stream=None):
    table = _freq_table(inv_freq, rotary_dim)
    _check(_lib.efim_decode_step_fp8_table(ctypes.byref(batch.c), _ptr(q), _ptr(k_new), _ptr(v_new),
                                           _ptr(k_cache), _ptr(v_cache), _ptr(out),
                                           table.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), int(rotary_dim),
                                           int(rope_interleaved), float(sm_scale), float(k_scale), float(v_scale),
                                           _ptr(workspace), int(workspace_bytes), _stream_ptr(stream)),
           "efim_decode_step_fp8_table")


def efim_extend_plan_items(batch):
    n = _lib.efim_extend_plan_items(ctypes.byref(batch.c), None, 0)
    if n < 0:
        raise EfimError(int(n), "efim_extend_plan_items")
    items = np.zeros(int(n), dtype=WORK_ITEM_DTYPE)
    if n:
        m = _lib.efim_extend_plan_items(ctypes.byref(batch.c), items.ctypes.data, int(n))
        assert m == n
    return items


def efim_set_tuning(key, value):
    _check(_lib.efim_set_tuning(int(key), int(value)), "efim_set_tuning")


def efim_set_kernel_events(start, stop):
    _check(_lib.efim_set_kernel_events(_ptr(start), _ptr(stop)), "efim_set_kernel_events")


def efim_status_string(status):
    return _lib.efim_status_string(int(status)).decode()


def efim_last_hip_error():
    return int(_lib.efim_last_hip_error())


def efim_version():
    return int(_lib.efim_version())


def raw_library():
    """The ctypes handle, for tests that exercise error returns of the C functions."""
    return _lib


class HipEvent:
    """A timing hipEvent_t created through the HIP runtime (used by the benchmark)."""
    _hip = None

    @classmethod
    def _rt(cls):
        if cls._hip is None:
            hip = ctypes.CDLL("libamdhip64.so")
            hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
            hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
            hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
            cls._hip = hip
        return cls._hip

    def __init__(self):
        self.handle = ctypes.c_void_p()
        rc = self._rt().hipEventCreate(ctypes.byref(self.handle))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)

    @property
    def ptr(self):
        return self.handle.value

    def record(self, stream=None):
        rc = self._rt().hipEventRecord(self.handle, _stream_ptr(stream))
        if rc != 0:
            raise RuntimeError("hipEventRecord failed: %d" % rc)

    def synchronize(self):
        rc = self._rt().hipEventSynchronize(self.handle)
        if rc != 0:
            raise RuntimeError("hipEventSynchronize failed: %d" % rc)

    def __del__(self):
        # (at interpreter shutdown the module globals may already be gone: then the process is
        # ending and the runtime reclaims the event)
        handle = getattr(self, "handle", None)
        if handle is not None and handle.value and self._hip is not None:
            self._hip.hipEventDestroy(handle)
            handle.value = None

    def elapsed_ms(self, end):
        ms = ctypes.c_float()
        rc = self._rt().hipEventElapsedTime(ctypes.byref(ms), self.handle, end.handle)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)


EFIM_ORDER_PSM, EFIM_ORDER_EFIM = 0, 1


def _tokens(seq):
    arr = np.ascontiguousarray(np.asarray(seq, dtype=np.int32).reshape(-1))
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), int(arr.size)


class SessionPool:
    """Owner of an efim_session_pool_t; the methods are the C calls of the same names."""

    def __init__(self, tok_p, tok_s, tok_m, reuse_granularity=1, always_psm=False):
        self.handle = _lib.efim_session_pool_create(int(tok_p), int(tok_s), int(tok_m), int(reuse_granularity),
                                                    int(bool(always_psm)))
        if not self.handle:
            raise EfimError(EFIM_ERR_INVALID_ARG, "efim_session_pool_create")

    def close(self):
        if self.handle:
            _lib.efim_session_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.close()

    def efim_session_transform(self, user, prefix, suffix):
        pre, pre_p, n_pre = _tokens(prefix)
        suf, suf_p, n_suf = _tokens(suffix)
        info = EfimPromptInfo()
        _check(_lib.efim_session_transform(self.handle, int(user), pre_p, n_pre, suf_p, n_suf, ctypes.byref(info)),
               "efim_session_transform")
        return {name: int(getattr(info, name)) for name, _ in EfimPromptInfo._fields_ if name != "reserved"}

    def efim_session_prompt(self, user):
        n = _lib.efim_session_prompt(self.handle, int(user), None, 0)
        if n < 0:
            raise EfimError(int(n), "efim_session_prompt")
        out = np.zeros(int(n), dtype=np.int32)
        if n:
            m = _lib.efim_session_prompt(self.handle, int(user), out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), int(n))
            assert m == n
        return out

    def efim_session_drop(self, user):
        rc = _lib.efim_session_drop(self.handle, int(user))
        if rc < 0:
            raise EfimError(int(rc), "efim_session_drop")
        return bool(rc)

    def efim_session_count(self):
        n = _lib.efim_session_count(self.handle)
        if n < 0:
            raise EfimError(int(n), "efim_session_count")
        return int(n)
