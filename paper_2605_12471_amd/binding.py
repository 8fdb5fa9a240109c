"""ctypes binding of include/kvfold.h: same names, argument marshalling only.

The library must have been built (``python -m paper_2605_12471_amd.build`` or
``__graft_entry__.build()``); loading fails loudly otherwise -- there is no
fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

KVFOLD_F32 = 0
KVFOLD_BF16 = 1
TUNE_SPLITS = 0
TUNE_UNITS_PER_WAVE = 1
TUNE_PAIR_UNITS = 2
TUNE_FUSED_APPEND = 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("KVFOLD_LIB_PATH") or os.path.join(_HERE, "_lib", "libkvfold.so")
_lib = None


class kvfold_config_t(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("n_layers", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("chunk_tokens", ctypes.c_int32),
        ("capacity_tokens", ctypes.c_int64),
        ("dtype", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
        ("device", ctypes.c_int32),
        ("kv_buffer", ctypes.c_void_p),
        ("kv_buffer_bytes", ctypes.c_size_t),
    ]


class kvfold_plan_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_workgroups", "n_splits", "units_per_wave", "tiles_per_split",
                                              "fused_append", "pair_units", "pair_order")]


class KvFoldError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {kvfold_status_string(status)} (status {status}, hip error {kvfold_last_hip_error()})")


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libkvfold.so and declare the prototypes of every exported entry point."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2605_12471_amd.build` "
            "(there is no non-HIP fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    cfgp = ctypes.POINTER(kvfold_config_t)
    lib.kvfold_cache_bytes_required.argtypes = [cfgp]
    lib.kvfold_cache_bytes_required.restype = ctypes.c_size_t
    lib.kvfold_cache_create.argtypes = [cfgp, ctypes.POINTER(vp)]
    lib.kvfold_cache_create.restype = ctypes.c_int
    lib.kvfold_step.argtypes = [vp, ctypes.c_int, vp, vp, vp, i64, vp, vp]
    lib.kvfold_step.restype = ctypes.c_int
    lib.kvfold_step_ex.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32, i64, vp, vp, vp]
    lib.kvfold_step_ex.restype = ctypes.c_int
    lib.kvfold_step_rope.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32, i64, vp, vp, vp, vp, vp]
    lib.kvfold_step_rope.restype = ctypes.c_int
    lib.kvfold_step_window.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32, i64, i32, i64, vp, vp, vp]
    lib.kvfold_step_window.restype = ctypes.c_int
    lib.kvfold_step_noalloc.argtypes = [vp, ctypes.c_int, vp, vp, vp, i32, i64, vp, vp, vp]
    lib.kvfold_step_noalloc.restype = ctypes.c_int
    lib.kvfold_cache_destroy.argtypes = [vp]
    lib.kvfold_cache_destroy.restype = ctypes.c_int
    lib.kvfold_cache_length.argtypes = [vp, ctypes.c_int]
    lib.kvfold_cache_length.restype = i64
    lib.kvfold_cache_view.argtypes = [vp, ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                      ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.kvfold_cache_view.restype = ctypes.c_int
    lib.kvfold_cache_truncate.argtypes = [vp, ctypes.c_int, i64]
    lib.kvfold_cache_truncate.restype = ctypes.c_int
    lib.kvfold_cache_set_length.argtypes = [vp, ctypes.c_int, i64]
    lib.kvfold_cache_set_length.restype = ctypes.c_int
    lib.kvfold_cache_set_storage_roundtrip.argtypes = [vp, i32]
    lib.kvfold_cache_set_storage_roundtrip.restype = ctypes.c_int
    lib.kvfold_cache_set_tuning.argtypes = [vp, i32, i32]
    lib.kvfold_cache_set_tuning.restype = ctypes.c_int
    lib.kvfold_cache_plan.argtypes = [vp, i32, i64, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.kvfold_cache_plan.restype = ctypes.c_int
    lib.kvfold_plan_for.argtypes = [ctypes.POINTER(kvfold_config_t), i32, i32, i64, i32, i64, ctypes.POINTER(kvfold_plan_t)]
    lib.kvfold_plan_for.restype = ctypes.c_int
    lib.kvfold_cache_profile_begin.argtypes = [vp, i32]
    lib.kvfold_cache_profile_begin.restype = ctypes.c_int
    dp = ctypes.POINTER(ctypes.c_double)
    lib.kvfold_cache_profile_end.argtypes = [vp, ctypes.POINTER(i32), dp, dp, dp]
    lib.kvfold_cache_profile_end.restype = ctypes.c_int
    lib.kvfold_status_string.argtypes = [ctypes.c_int]
    lib.kvfold_status_string.restype = ctypes.c_char_p
    lib.kvfold_measure_peaks.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.kvfold_measure_peaks.restype = ctypes.c_int
    lib.kvfold_last_hip_error.argtypes = []
    lib.kvfold_last_hip_error.restype = ctypes.c_int
    _lib = lib
    return lib


# ---------------------------------------------------------------------------------------------
# Functions with the header's names.  Pointers are plain integers (e.g. torch's data_ptr()).
# Each returns the library's status code (or value) untouched.
# ---------------------------------------------------------------------------------------------
def make_config(n_layers, n_q_heads, n_kv_heads, head_dim, chunk_tokens, capacity_tokens, dtype,
                softmax_scale=0.0, device=0, kv_buffer=None, kv_buffer_bytes=0) -> kvfold_config_t:
    return kvfold_config_t(ctypes.sizeof(kvfold_config_t), n_layers, n_q_heads, n_kv_heads, head_dim, chunk_tokens,
                           capacity_tokens, dtype, softmax_scale, device, kv_buffer, kv_buffer_bytes)


def kvfold_cache_bytes_required(cfg: kvfold_config_t) -> int:
    return int(load_library().kvfold_cache_bytes_required(ctypes.byref(cfg)))


def kvfold_cache_create(cfg: Optional[kvfold_config_t]):
    """Returns (status, handle); handle is None on error."""
    h = ctypes.c_void_p()
    rc = load_library().kvfold_cache_create(ctypes.byref(cfg) if cfg is not None else None, ctypes.byref(h))
    return rc, (h if rc == 0 else None)


def kvfold_step(cache, layer, q, k_new, v_new, pos_offset, out, stream=0) -> int:
    return load_library().kvfold_step(cache, layer, q, k_new, v_new, pos_offset, out, stream)


def kvfold_step_ex(cache, layer, q, k_new, v_new, n_tokens, pos_offset, out, lse=None, stream=0) -> int:
    return load_library().kvfold_step_ex(cache, layer, q, k_new, v_new, n_tokens, pos_offset, out, lse, stream)


def kvfold_step_rope(cache, layer, q, k_new, v_new, n_tokens, pos_offset, rope_cos, rope_sin, out, lse=None,
                     stream=0) -> int:
    return load_library().kvfold_step_rope(cache, layer, q, k_new, v_new, n_tokens, pos_offset, rope_cos, rope_sin,
                                           out, lse, stream)


def kvfold_step_window(cache, layer, q, k_new, v_new, n_tokens, pos_offset, n_sink, window, out, lse=None, stream=0) -> int:
    return load_library().kvfold_step_window(cache, layer, q, k_new, v_new, n_tokens, pos_offset, n_sink, window,
                                             out, lse, stream)


def kvfold_step_noalloc(cache, layer, q, k_new, v_new, n_tokens, pos_offset, out, lse=None, stream=0) -> int:
    return load_library().kvfold_step_noalloc(cache, layer, q, k_new, v_new, n_tokens, pos_offset, out, lse, stream)


def kvfold_cache_destroy(cache) -> int:
    return load_library().kvfold_cache_destroy(cache)


def kvfold_cache_length(cache, layer) -> int:
    return int(load_library().kvfold_cache_length(cache, layer))


def kvfold_cache_view(cache, layer):
    """Returns (status, k_ptr, v_ptr, row_stride_elems, head_stride_elems)."""
    k, v = ctypes.c_void_p(), ctypes.c_void_p()
    rs, hs = ctypes.c_int64(), ctypes.c_int64()
    rc = load_library().kvfold_cache_view(cache, layer, ctypes.byref(k), ctypes.byref(v), ctypes.byref(rs),
                                          ctypes.byref(hs))
    return rc, k.value, v.value, rs.value, hs.value


def kvfold_cache_truncate(cache, layer, new_len) -> int:
    return load_library().kvfold_cache_truncate(cache, layer, new_len)


def kvfold_cache_set_length(cache, layer, new_len) -> int:
    return load_library().kvfold_cache_set_length(cache, layer, new_len)


def kvfold_cache_set_storage_roundtrip(cache, n_bits) -> int:
    return load_library().kvfold_cache_set_storage_roundtrip(cache, n_bits)


def kvfold_cache_set_tuning(cache, knob, value) -> int:
    return load_library().kvfold_cache_set_tuning(cache, knob, value)


def kvfold_cache_plan(cache, n_tokens, len_after):
    """Returns (status, n_workgroups, n_splits)."""
    w, s = ctypes.c_int32(), ctypes.c_int32()
    rc = load_library().kvfold_cache_plan(cache, n_tokens, len_after, ctypes.byref(w), ctypes.byref(s))
    return rc, w.value, s.value


def kvfold_plan_for(cfg, n_compute_units, n_tokens, len_after, n_sink=0, window=0):
    """Host-only.  Returns (status, kvfold_plan_t)."""
    pl = kvfold_plan_t()
    rc = load_library().kvfold_plan_for(ctypes.byref(cfg) if cfg is not None else None, n_compute_units, n_tokens, len_after,
                                        n_sink, window, ctypes.byref(pl))
    return rc, pl


def kvfold_cache_profile_begin(cache, max_steps) -> int:
    return load_library().kvfold_cache_profile_begin(cache, max_steps)


def kvfold_cache_profile_end(cache):
    """Returns (status, n_steps, append_ms, attention_ms, merge_ms)."""
    n = ctypes.c_int32()
    a, t, m = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    rc = load_library().kvfold_cache_profile_end(cache, ctypes.byref(n), ctypes.byref(a), ctypes.byref(t),
                                                 ctypes.byref(m))
    return rc, n.value, a.value, t.value, m.value


def kvfold_status_string(status: int) -> str:
    return load_library().kvfold_status_string(status).decode()


def kvfold_measure_peaks(device=0, mfma=True, hbm=True):
    """(status, bf16 matrix-instruction TFLOP/s or None, HBM read GB/s or None) of the GPU `device`."""
    t, g = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = load_library().kvfold_measure_peaks(device, ctypes.byref(t) if mfma else None, ctypes.byref(g) if hbm else None)
    return rc, (t.value if mfma and rc == 0 else None), (g.value if hbm and rc == 0 else None)


def kvfold_last_hip_error() -> int:
    return int(load_library().kvfold_last_hip_error())


# ---------------------------------------------------------------------------------------------
# Convenience wrapper for torch callers (still marshalling only).
# ---------------------------------------------------------------------------------------------
class KvFoldCache:
    """Owns one library cache handle; ``step`` takes torch tensors on the cache's device."""

    def __init__(self, n_layers, n_q_heads, n_kv_heads, head_dim, chunk_tokens, capacity_tokens, dtype="bf16",
                 softmax_scale=0.0, device=0):
        self.dtype_name = dtype
        self.cfg = make_config(n_layers, n_q_heads, n_kv_heads, head_dim, chunk_tokens, capacity_tokens,
                               {"f32": KVFOLD_F32, "bf16": KVFOLD_BF16}[dtype], softmax_scale, device)
        rc, self.handle = kvfold_cache_create(self.cfg)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_create")

    def close(self):
        if getattr(self, "handle", None) is not None:
            rc = kvfold_cache_destroy(self.handle)
            self.handle = None
            if rc:
                raise KvFoldError(rc, "kvfold_cache_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _stream(self, stream):
        if stream is not None:
            return stream
        import torch
        return torch.cuda.current_stream().cuda_stream

    def _check(self, name, t, shape, dtype=None):
        """Marshalling validation: the kernels trust shapes and element types, so a mismatch must stop here."""
        import torch
        want = dtype or (torch.float32 if self.dtype_name == "f32" else torch.bfloat16)
        if not (t.is_cuda and t.device.index == self.cfg.device):
            raise ValueError(f"{name}: expected a tensor on cuda:{self.cfg.device}, got {t.device}")
        if t.dtype != want:
            raise ValueError(f"{name}: expected dtype {want}, got {t.dtype}")
        if tuple(t.shape) != tuple(shape):
            raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
        if not t.is_contiguous():
            raise ValueError(f"{name}: expected a contiguous tensor")

    def step(self, layer, q, k_new, v_new, out, pos_offset=None, lse=None, stream=None, rope=None, window=None,
             noalloc=False):
        """Enqueue one fold step; q/k_new/v_new/out (and lse) are contiguous device tensors.  rope = (cos, sin),
        fp32 device tensors [n][head_dim/2]: q and k_new are unrotated and the step rotates them.  window =
        (n_sink, window): the sink + sliding-window step.  noalloc: through kvfold_step_noalloc."""
        import torch
        c = self.cfg
        n = q.shape[0] if q.dim() == 3 else -1
        pos = self.length(layer) if pos_offset is None else pos_offset
        self._check("q", q, (n, c.n_q_heads, c.head_dim))
        self._check("out", out, (n, c.n_q_heads, c.head_dim))
        self._check("k_new", k_new, (n, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (n, c.n_kv_heads, c.head_dim))
        if lse is not None:
            self._check("lse", lse, (c.n_q_heads, n), torch.float32)
        lse_ptr = lse.data_ptr() if lse is not None else None
        if sum(x is not None and x is not False for x in (rope, window, noalloc)) > 1:
            raise ValueError("rope, window and noalloc are separate entry points")
        if window is not None:
            n_sink, win = window
            rc = kvfold_step_window(self.handle, layer, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), n, pos,
                                    n_sink, win, out.data_ptr(), lse_ptr, self._stream(stream))
            if rc:
                raise KvFoldError(rc, "kvfold_step_window")
            return out
        if rope is None:
            fn, name = (kvfold_step_noalloc, "kvfold_step_noalloc") if noalloc else (kvfold_step_ex, "kvfold_step_ex")
            rc = fn(self.handle, layer, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), n, pos,
                    out.data_ptr(), lse_ptr, self._stream(stream))
            if rc:
                raise KvFoldError(rc, name)
            return out
        cos, sin = rope
        self._check("rope cos", cos, (n, c.head_dim // 2), torch.float32)
        self._check("rope sin", sin, (n, c.head_dim // 2), torch.float32)
        rc = kvfold_step_rope(self.handle, layer, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), n, pos,
                              cos.data_ptr(), sin.data_ptr(), out.data_ptr(), lse_ptr, self._stream(stream))
        if rc:
            raise KvFoldError(rc, "kvfold_step_rope")
        return out

    def bytes_required(self) -> int:
        return kvfold_cache_bytes_required(self.cfg)

    def length(self, layer=0) -> int:
        n = kvfold_cache_length(self.handle, layer)
        if n < 0:
            raise KvFoldError(n, "kvfold_cache_length")
        return n

    def truncate(self, layer, new_len):
        rc = kvfold_cache_truncate(self.handle, layer, new_len)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_truncate")

    def set_length(self, layer, new_len):
        rc = kvfold_cache_set_length(self.handle, layer, new_len)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_set_length")

    def set_storage_roundtrip(self, n_bits):
        rc = kvfold_cache_set_storage_roundtrip(self.handle, n_bits)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_set_storage_roundtrip")

    def set_tuning(self, knob, value):
        rc = kvfold_cache_set_tuning(self.handle, knob, value)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_set_tuning")

    def plan(self, n_tokens, len_after):
        rc, w, s = kvfold_cache_plan(self.handle, n_tokens, len_after)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_plan")
        return w, s

    def profile_begin(self, max_steps):
        rc = kvfold_cache_profile_begin(self.handle, max_steps)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_profile_begin")

    def profile_end(self):
        """(n_steps, append_ms, attention_ms, merge_ms) summed over the profiled steps."""
        rc, n, a, t, m = kvfold_cache_profile_end(self.handle)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_profile_end")
        return n, a, t, m

    def view(self, layer=0):
        """(K, V) device tensors [Hkv][capacity][d] aliasing the cache rows of ``layer`` (no copy)."""
        import torch
        rc, k, v, rs, hs = kvfold_cache_view(self.handle, layer)
        if rc:
            raise KvFoldError(rc, "kvfold_cache_view")
        c = self.cfg
        es = 4 if self.dtype_name == "f32" else 2

        def wrap(ptr):
            class _Holder:  # device memory described by pointer + shape; torch aliases it, nothing is copied
                __cuda_array_interface__ = {"shape": (c.n_kv_heads, c.capacity_tokens, c.head_dim),
                                            "typestr": "<f4" if es == 4 else "<i2", "data": (ptr, False),
                                            "version": 3}
            t = torch.as_tensor(_Holder(), device=f"cuda:{c.device}")
            return t if es == 4 else t.view(torch.bfloat16)

        return wrap(k), wrap(v)
