"""fp64 CPU oracle for the KV-Fold fold step -- TEST INFRASTRUCTURE, not product code.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module; the HIP library never does and shares no
code with it.

What it holds
-------------
* :class:`OracleCache` / :meth:`OracleCache.step` -- the fold step of the
  paper's Sec. 2 ("KV-Fold"; recurrence in "A recurrent view"): append the
  chunk's K/V rows to a per-layer carried cache, then let the chunk's queries
  attend to every cached row up to and including their own position.  The
  arithmetic is the plain definition, done row by row in ``kvfold_oracle.c``.
* ``OracleCache.step(..., n_sink=, window=)`` -- the same step under the sink + sliding-window mask of
  the streaming baseline the paper compares with (Sec. 6), ``kvfold_oracle_attend_rows_window``.
* :func:`monolithic_causal_attention` -- the paper's FULL condition (Sec. 2,
  "Three reference conditions"): one causal pass over all T tokens, written
  independently in numpy by materialising the T x T masked score matrix.  It
  exists to pin the fold (any chunking == one monolithic pass).

Readings of the paper taken here (the paper is silent on all of them):
contiguous grouped-query mapping (query head h -> KV head h // (Hq/Hkv)),
diagonal-inclusive causal mask, softmax scale 1/sqrt(d) unless given,
queries/keys used as handed in (already rotated); :func:`rope` is the rotation
itself for the entry point that takes them unrotated (half-split pairing, fp32).

Parity pins: tests/test_oracle_pins.py (fold invariant vs the monolithic pass,
brute-force python loops, torch's fp64 scaled_dot_product_attention, closed
forms, invariances).  No function here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvfold_oracle.c")
_LIB = os.path.join(_HERE, "libkvfold_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, -O3). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i64 = ctypes.c_int64
            vp = ctypes.c_void_p
            lib.kvfold_oracle_append_bytes.argtypes = [vp, i64, i64, i64, i64, vp, i64, i64]
            lib.kvfold_oracle_append_bytes.restype = ctypes.c_int
            lib.kvfold_oracle_attend_rows.argtypes = [vp, vp, i64, i64, i64, vp, i64, i64, i64,
                                                      ctypes.c_double, vp, i64, vp, vp, vp]
            lib.kvfold_oracle_attend_rows.restype = ctypes.c_int
            lib.kvfold_oracle_attend_rows_window.argtypes = [vp, vp, i64, i64, i64, vp, i64, i64, i64,
                                                             ctypes.c_double, i64, i64, vp, i64, vp, vp, vp]
            lib.kvfold_oracle_attend_rows_window.restype = ctypes.c_int
            lib.kvfold_oracle_threads.restype = ctypes.c_int
            lib.kvfold_oracle_rope_f32.argtypes = [vp, i64, i64, i64, vp, vp, vp]
            lib.kvfold_oracle_rope_f32.restype = ctypes.c_int
            _lib = lib
    return _lib


def threads() -> int:
    """Number of host threads the C oracle uses."""
    return int(_load().kvfold_oracle_threads())


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even of fp32 values to bfloat16 bit patterns (finite values and infinities)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotary embedding of x [rows][heads][d] (fp32) by the angles cos/sin [rows][d/2] of the rows'
    absolute positions (Sec. 2: positions continue from tC), half-split pairing, fp32 with the
    rounding points of ``kvfold_oracle_rope_f32``.  Returns fp32; a bf16 fold stores
    ``f32_to_bf16_bits`` of it."""
    x = np.ascontiguousarray(x, np.float32)
    rows, heads, d = x.shape
    cos = np.ascontiguousarray(cos, np.float32)
    sin = np.ascontiguousarray(sin, np.float32)
    assert cos.shape == (rows, d // 2) and sin.shape == (rows, d // 2)
    out = np.empty_like(x)
    rc = _load().kvfold_oracle_rope_f32(_ptr(x), rows, heads, d, _ptr(cos), _ptr(sin), _ptr(out))
    if rc:
        raise ValueError("head_dim must be even")
    return out


def storage_roundtrip(bits16: np.ndarray, n_bits: int) -> np.ndarray:
    """The paper's storage perturbation (Sec. 8, Discussion: a per-step quantisation round trip
    bf16 -> intN -> bf16 of the carried cache), applied to rows as they join the cache.  The paper gives
    no quantiser; the reading taken: one group = the d elements of one (token, KV head) row, symmetric,
    scale = max|x| / (2^(N-1) - 1), code = round-half-even(x / scale) clamped to +-(2^(N-1) - 1),
    value = code * scale, all in fp32, stored as bf16 (RNE).  An all-zero row stays zero.
    bits16: [..., d] bf16 bit patterns; returns the same shape."""
    assert n_bits in (4, 8)
    x = bf16_bits_to_f32(bits16)
    qmax = np.float32(2 ** (n_bits - 1) - 1)
    amax = np.abs(x).max(axis=-1, keepdims=True).astype(np.float32)
    scale = (amax / qmax).astype(np.float32)
    safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    code = np.clip(np.rint((x / safe).astype(np.float32)), -qmax, qmax).astype(np.float32)
    y = (code * safe).astype(np.float32)
    y = np.where(scale > 0, y, np.float32(0.0)).astype(np.float32)
    return f32_to_bf16_bits(y).reshape(bits16.shape)


class OracleCache:
    """Carried KV cache of ONE layer plus the fold step on it.

    ``store_dtype`` is the numpy dtype of the *stored* elements (np.float32,
    np.float64, or np.uint16 holding bfloat16 bit patterns).  The stored bits
    are what the device cache must equal byte for byte; the fp64 widening of
    those bits is what attention runs on.
    """

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, capacity: int,
                 scale: float | None = None, store_dtype=np.float64):
        if n_q_heads % n_kv_heads:
            raise ValueError("Hq must be a multiple of Hkv")
        self.Hq, self.Hkv, self.d, self.cap = n_q_heads, n_kv_heads, head_dim, capacity
        self.scale = float(scale) if scale else 1.0 / float(np.sqrt(head_dim))
        self.len = 0
        self.store_dtype = np.dtype(store_dtype)
        self.k_bits = np.zeros((n_kv_heads, capacity, head_dim), self.store_dtype)
        self.v_bits = np.zeros((n_kv_heads, capacity, head_dim), self.store_dtype)
        self.K = np.zeros((n_kv_heads, capacity, head_dim), np.float64)
        self.V = np.zeros((n_kv_heads, capacity, head_dim), np.float64)

    # -- widening of stored elements to fp64 (exact for every supported type)
    def _widen(self, bits: np.ndarray) -> np.ndarray:
        if self.store_dtype == np.uint16:  # bfloat16 bit pattern -> upper half of a float32
            return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        return bits.astype(np.float64)

    def append(self, k_new: np.ndarray, v_new: np.ndarray) -> None:
        """Cache carry: rows [len, len+C) := the chunk's rows; older rows untouched."""
        lib = _load()
        C = k_new.shape[0]
        for cache_bits, cache64, new in ((self.k_bits, self.K, k_new), (self.v_bits, self.V, v_new)):
            new = np.ascontiguousarray(new, self.store_dtype)
            assert new.shape == (C, self.Hkv, self.d)
            rc = lib.kvfold_oracle_append_bytes(_ptr(cache_bits), self.Hkv, self.cap, self.d, self.len,
                                                _ptr(new), C, self.store_dtype.itemsize)
            if rc:
                raise ValueError("append beyond capacity")
            wide = np.ascontiguousarray(self._widen(new))
            rc = lib.kvfold_oracle_append_bytes(_ptr(cache64), self.Hkv, self.cap, self.d, self.len,
                                                _ptr(wide), C, 8)
            assert rc == 0
        self.len += C

    def step(self, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, pos_offset: int,
             rows=None, want_weights: bool = False, n_sink: int = 0, window: int | None = None):
        """One fold step. ``q`` is [C][Hq][d] fp64 (already widened by the caller).

        ``pos_offset`` must equal the current cache length (positions continue
        from tC, Sec. 2).  ``rows`` selects chunk rows to evaluate (default all).
        Returns (out [nrows][Hq][d], lse [nrows][Hq]) and, if asked, the softmax
        weights [nrows][Hq][len_after].  ``window`` (with ``n_sink``) selects the sink + sliding-window
        mask of the streaming baseline (Sec. 6): the append is the same, the row at absolute position p
        attends to keys j < n_sink and p - window < j <= p only.
        """
        if pos_offset != self.len:
            raise ValueError(f"pos_offset {pos_offset} != cache length {self.len}")
        len_prev = self.len
        self.append(k_new, v_new)
        return self.attend(q, len_prev, rows, want_weights, n_sink, window)

    def attend(self, q: np.ndarray, len_prev: int, rows=None, want_weights: bool = False,
               n_sink: int = 0, window: int | None = None):
        """Attention of chunk rows against the cache that already holds the chunk."""
        lib = _load()
        q = np.ascontiguousarray(q, np.float64)
        C = q.shape[0]
        assert q.shape == (C, self.Hq, self.d)
        rows = np.arange(C, dtype=np.int64) if rows is None else np.ascontiguousarray(rows, np.int64)
        n = len(rows)
        out = np.empty((n, self.Hq, self.d), np.float64)
        lse = np.empty((n, self.Hq), np.float64)
        w = np.empty((n, self.Hq, len_prev + C), np.float64) if want_weights else None
        if window is None:
            rc = lib.kvfold_oracle_attend_rows(_ptr(self.K), _ptr(self.V), self.Hkv, self.cap, self.d, _ptr(q),
                                               C, self.Hq, len_prev, self.scale, _ptr(rows), n,
                                               _ptr(out), _ptr(lse), _ptr(w) if want_weights else None)
        else:
            rc = lib.kvfold_oracle_attend_rows_window(_ptr(self.K), _ptr(self.V), self.Hkv, self.cap, self.d, _ptr(q),
                                                      C, self.Hq, len_prev, self.scale, int(n_sink), int(window),
                                                      _ptr(rows), n, _ptr(out), _ptr(lse),
                                                      _ptr(w) if want_weights else None)
        if rc:
            raise ValueError(f"oracle attend failed rc={rc}")
        return (out, lse, w) if want_weights else (out, lse)


def fold(Q: np.ndarray, K: np.ndarray, V: np.ndarray, chunk_sizes, n_kv_heads: int | None = None,
         scale: float | None = None, n_sink: int = 0, window: int | None = None):
    """Left fold over chunks (Sec. 2: foldl(F, (empty, empty), [x_0 .. x_{N-1}])).

    Q [T][Hq][d], K/V [T][Hkv][d] fp64; ``chunk_sizes`` sums to T.  Returns
    (out [T][Hq][d], lse [T][Hq]).  ``window`` / ``n_sink``: every step under the sink + sliding-window mask.
    """
    T, Hq, d = Q.shape
    Hkv = K.shape[1] if n_kv_heads is None else n_kv_heads
    assert sum(chunk_sizes) == T
    cache = OracleCache(Hq, Hkv, d, T, scale)
    outs, lses, pos = [], [], 0
    for C in chunk_sizes:
        o, l = cache.step(Q[pos:pos + C], K[pos:pos + C], V[pos:pos + C], pos, n_sink=n_sink, window=window)
        outs.append(o)
        lses.append(l)
        pos += C
    return np.concatenate(outs, 0), np.concatenate(lses, 0)


def monolithic_causal_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float | None = None):
    """FULL condition: one causal pass over the whole sequence, T x T scores materialised.

    Independent numpy code path (no C, no chunks).  Q [T][Hq][d], K/V [T][Hkv][d].
    Returns (out [T][Hq][d], lse [T][Hq]).
    """
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    scale = float(scale) if scale else 1.0 / float(np.sqrt(d))
    out = np.empty((T, Hq, d), np.float64)
    lse = np.empty((T, Hq), np.float64)
    future = np.triu(np.ones((T, T), bool), k=1)  # key index > query index
    for h in range(Hq):
        g = h // G
        S = (Q[:, h, :] @ K[:, g, :].T) * scale
        S[future] = -np.inf
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        l = E.sum(axis=1, keepdims=True)
        out[:, h, :] = (E / l) @ V[:, g, :]
        lse[:, h] = (m + np.log(l))[:, 0]
    return out, lse
