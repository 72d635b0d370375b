"""CPU oracle for the LightTransfer hot path -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Thin ctypes wrapper over ``lt_oracle.c`` (plain C, fp64).  Only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package; the GPU
library and its Python binding never do, and nothing here imports them.

All tensors are numpy arrays; bf16 data travels as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lt_oracle.c")
# LT_ORACLE_LIBRARY names another build of lt_oracle.c to load instead (the sanitizer build the test-suite makes)
_LIB = os.environ.get("LT_ORACLE_LIBRARY") or os.path.join(_HERE, "liblt_oracle.so")

MODE_FULL = 0
MODE_LAZY = 1
RECENT_PER_QUERY = 0
RECENT_FIXED = 1


def build(force: bool = False) -> str:
    """Compile lt_oracle.c with gcc when the library is missing or older than its source."""
    if os.environ.get("LT_ORACLE_LIBRARY"):
        return _LIB                             # somebody else's build: used as it is
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int)
        u8p = ctypes.POINTER(ctypes.c_ubyte)
        c_int, c_i64, c_f64 = ctypes.c_int, ctypes.c_int64, ctypes.c_double
        lib.lto_decode_attn.argtypes = [u16p, u16p, u16p, c_int, c_int, c_int, c_int, c_i64,
                                        c_int, c_i64, c_i64, c_f64, f64p, f64p, f64p]
        lib.lto_decode_attn.restype = c_int
        for fn in (lib.lto_lazy_ratio, lib.lto_lazy_ratio_lse):
            fn.argtypes = [u16p, u16p, c_int, c_int, c_int, c_int, c_i64, c_int,
                           c_i64, c_i64, c_f64, c_int, f64p, f64p, f64p]
            fn.restype = c_int
        lib.lto_lazy_ratio_from_lse.argtypes = [u16p, u16p, f64p, c_int, c_int, c_int, c_int, c_i64, c_int,
                                                c_i64, c_i64, c_f64, c_int, f64p, f64p, f64p]
        lib.lto_lazy_ratio_from_lse.restype = c_int
        lib.lto_prefill_attn.argtypes = [u16p, u16p, u16p, c_int, c_int, c_int, c_int, c_i64,
                                         c_int, c_i64, c_i64, c_f64, f64p, f64p, f64p]
        lib.lto_prefill_attn.restype = c_int
        lib.lto_select_lazy.argtypes = [f64p, c_int, c_int, u8p, i32p]
        lib.lto_select_lazy.restype = c_int
        lib.lto_select_lazy_queue.argtypes = [f64p, c_int, c_int, u8p, i32p]
        lib.lto_select_lazy_queue.restype = c_int
        lib.lto_preselect_lazy.argtypes = [u8p, c_int, c_int, c_int, i32p, u8p]
        lib.lto_preselect_lazy.restype = c_int
        lib.lto_num_threads.restype = c_int
        lib.lto_set_num_threads.argtypes = [c_int]
        _lib = lib
    return _lib


def _u16(a, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 data must be passed as uint16 bit patterns, got %s" % a.dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (tuple(shape), a.shape))
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check(status, what):
    if status != 0:
        raise ValueError("%s: oracle rejected its arguments (status %d)" % (what, status))


def num_threads() -> int:
    return int(_load().lto_num_threads())


def set_num_threads(n: int) -> None:
    _load().lto_set_num_threads(int(n))


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns, as float64 (for tests that need the numbers)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even) and return the bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + 0x7FFF + ((u >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def decode_attn(q, K, V, mode, w_sink=0, w_recent=0, scale=None, return_probs=False):
    """Decode attention of the newest token over a layer's whole history.

    q [B,Hq,d], K/V [B,Hkv,T,d] as uint16 bf16 bits.  Returns (out [B,Hq,d], lse [B,Hq])
    as float64, plus probs [B,Hq,T] when ``return_probs``.
    """
    lib = _load()
    q = _u16(q)
    B, Hq, d = q.shape
    K = _u16(K)
    _, Hkv, T, _ = K.shape
    K = _u16(K, (B, Hkv, T, d))
    V = _u16(V, (B, Hkv, T, d))
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    probs = np.empty((B, Hq, T), dtype=np.float64) if return_probs else None
    st = lib.lto_decode_attn(_ptr(q, ctypes.c_uint16), _ptr(K, ctypes.c_uint16), _ptr(V, ctypes.c_uint16),
                             B, Hq, Hkv, d, T, int(mode), int(w_sink), int(w_recent), float(scale),
                             _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double),
                             _ptr(probs, ctypes.c_double) if return_probs else None)
    _check(st, "decode_attn")
    return (out, lse, probs) if return_probs else (out, lse)


def _ratio_call(fn, q_last, K, w_sink, w_recent, scale, recent_mode):
    q_last = _u16(q_last)
    B, Hq, w, d = q_last.shape
    K = _u16(K)
    _, Hkv, n, _ = K.shape
    K = _u16(K, (B, Hkv, n, d))
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    per = np.empty((B, Hq, w), dtype=np.float64)
    r_seq = np.empty((B,), dtype=np.float64)
    r = np.empty((1,), dtype=np.float64)
    st = fn(_ptr(q_last, ctypes.c_uint16), _ptr(K, ctypes.c_uint16), B, Hq, Hkv, d, n, w,
            int(w_sink), int(w_recent), float(scale), int(recent_mode),
            _ptr(per, ctypes.c_double), _ptr(r_seq, ctypes.c_double), _ptr(r, ctypes.c_double))
    _check(st, "lazy_ratio")
    return per, r_seq, float(r[0])


def lazy_ratio(q_last, K, w_sink, w_recent, scale=None, recent_mode=RECENT_PER_QUERY):
    """Eq. 1 form.  Returns (rho [B,Hq,w], r_seq [B], r)."""
    return _ratio_call(_load().lto_lazy_ratio, q_last, K, w_sink, w_recent, scale, recent_mode)


def lazy_ratio_lse(q_last, K, w_sink, w_recent, scale=None, recent_mode=RECENT_PER_QUERY):
    """Table 1 form.  Returns (log_rho [B,Hq,w], r_seq [B], r)."""
    return _ratio_call(_load().lto_lazy_ratio_lse, q_last, K, w_sink, w_recent, scale, recent_mode)


def lazy_ratio_from_lse(q_last, K, lse_rows, w_sink, w_recent, scale=None, recent_mode=RECENT_PER_QUERY):
    """Table 1 with the prefill's log-sum-exp supplied: lse_rows [B,Hq,w] (natural log) of the causal rows
    n-w..n-1.  Returns (log_rho [B,Hq,w], r_seq [B], r)."""
    q_last = _u16(q_last)
    B, Hq, w, d = q_last.shape
    K = _u16(K)
    _, Hkv, n, _ = K.shape
    K = _u16(K, (B, Hkv, n, d))
    lse_rows = np.ascontiguousarray(lse_rows, dtype=np.float64)
    if lse_rows.shape != (B, Hq, w):
        raise ValueError(f"lse_rows has shape {lse_rows.shape}, expected {(B, Hq, w)}")
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    per = np.empty((B, Hq, w), dtype=np.float64)
    r_seq = np.empty((B,), dtype=np.float64)
    r = np.empty((1,), dtype=np.float64)
    st = _load().lto_lazy_ratio_from_lse(_ptr(q_last, ctypes.c_uint16), _ptr(K, ctypes.c_uint16),
                                         _ptr(lse_rows, ctypes.c_double), B, Hq, Hkv, d, n, w,
                                         int(w_sink), int(w_recent), float(scale), int(recent_mode),
                                         _ptr(per, ctypes.c_double), _ptr(r_seq, ctypes.c_double), _ptr(r, ctypes.c_double))
    _check(st, "lazy_ratio_from_lse")
    return per, r_seq, float(r[0])


def prefill_attn(Q, K, V, mode, w_sink=0, w_recent=0, scale=None, return_absw=False):
    """Prefill attention over a whole prompt.  Q [B,Hq,n,d], K/V [B,Hkv,n,d] as uint16 bf16 bits.
    Returns (out [B,Hq,n,d], lse [B,Hq,n]) as float64, plus absw [B,Hq,n,d] = sum_j p_j |V_j| when asked."""
    Q = _u16(Q)
    B, Hq, n, d = Q.shape
    K = _u16(K)
    Hkv = K.shape[1]
    K = _u16(K, (B, Hkv, n, d))
    V = _u16(V, (B, Hkv, n, d))
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((B, Hq, n, d), dtype=np.float64)
    lse = np.empty((B, Hq, n), dtype=np.float64)
    absw = np.empty((B, Hq, n, d), dtype=np.float64) if return_absw else None
    st = _load().lto_prefill_attn(_ptr(Q, ctypes.c_uint16), _ptr(K, ctypes.c_uint16), _ptr(V, ctypes.c_uint16),
                                  B, Hq, Hkv, d, n, int(mode), int(w_sink), int(w_recent), float(scale),
                                  _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double),
                                  _ptr(absw, ctypes.c_double) if return_absw else None)
    _check(st, "prefill_attn")
    return (out, lse, absw) if return_absw else (out, lse)


def select_lazy(ratios, n_lazy):
    """Top-n_lazy layers by (ratio descending, index ascending).  Returns (is_lazy u8 [L], order i32 [L])."""
    r = np.ascontiguousarray(ratios, dtype=np.float64)
    L = r.shape[0]
    is_lazy = np.zeros((L,), dtype=np.uint8)
    order = np.zeros((L,), dtype=np.int32)
    st = _load().lto_select_lazy(_ptr(r, ctypes.c_double), L, int(n_lazy),
                                 _ptr(is_lazy, ctypes.c_ubyte), _ptr(order, ctypes.c_int))
    _check(st, "select_lazy")
    return is_lazy, order


def select_lazy_queue(ratios, n_lazy):
    """Priority-queue simulation.  Returns (is_lazy u8 [L], pop_step i32 [L])."""
    r = np.ascontiguousarray(ratios, dtype=np.float64)
    L = r.shape[0]
    is_lazy = np.zeros((L,), dtype=np.uint8)
    pop_step = np.zeros((L,), dtype=np.int32)
    st = _load().lto_select_lazy_queue(_ptr(r, ctypes.c_double), L, int(n_lazy),
                                       _ptr(is_lazy, ctypes.c_ubyte), _ptr(pop_step, ctypes.c_int))
    _check(st, "select_lazy_queue")
    return is_lazy, pop_step


def preselect_lazy(sets, n_lazy):
    """LightTransfer-Train pre-selection.  sets uint8 [S, L]; returns (is_lazy u8 [L], count i32 [L])."""
    m = np.ascontiguousarray(np.asarray(sets) != 0, dtype=np.uint8)
    S, L = m.shape
    is_lazy = np.zeros((L,), dtype=np.uint8)
    count = np.zeros((L,), dtype=np.int32)
    st = _load().lto_preselect_lazy(_ptr(m, ctypes.c_ubyte), S, L, int(n_lazy), _ptr(count, ctypes.c_int),
                                    _ptr(is_lazy, ctypes.c_ubyte))
    _check(st, "preselect_lazy")
    return is_lazy, count


class History:
    """Positional KV history of a layer stack: append keeps every token, nothing else.

    The reduced cache of a lazy layer is never built here; decode() applies the
    streaming set to the whole history instead.
    """

    def __init__(self, n_layers, is_lazy, w_sink, w_recent, scale=None):
        self.n_layers = int(n_layers)
        self.is_lazy = [bool(x) for x in is_lazy]
        if len(self.is_lazy) != self.n_layers:
            raise ValueError("is_lazy must have one entry per layer")
        self.w_sink, self.w_recent, self.scale = int(w_sink), int(w_recent), scale
        self.K = [None] * self.n_layers
        self.V = [None] * self.n_layers

    def append(self, layer, k_new, v_new):
        k_new, v_new = _u16(k_new), _u16(v_new)
        if k_new.shape != v_new.shape or k_new.ndim != 4:
            raise ValueError("k_new and v_new must both be [B,Hkv,n_new,d]")
        if self.K[layer] is None:
            self.K[layer], self.V[layer] = k_new.copy(), v_new.copy()
        else:
            self.K[layer] = np.concatenate([self.K[layer], k_new], axis=2)
            self.V[layer] = np.concatenate([self.V[layer], v_new], axis=2)

    def length(self, layer):
        return 0 if self.K[layer] is None else int(self.K[layer].shape[2])

    def decode(self, layer, q):
        mode = MODE_LAZY if self.is_lazy[layer] else MODE_FULL
        return decode_attn(q, self.K[layer], self.V[layer], mode, self.w_sink, self.w_recent, self.scale)
