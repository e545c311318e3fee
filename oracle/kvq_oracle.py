"""ctypes/numpy front end of the C oracle (oracle/kvq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the CPU-baseline leg of the
benchmark.  The GPU library never imports or calls anything in this package.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

# KVQ_ORACLE_LIB: load this build of the oracle instead (the test that plants mistakes in a copy of
# the C source and checks that the pins notice uses it; nothing else sets it)
_lib = C.CDLL(os.environ.get("KVQ_ORACLE_LIB") or _build.build())

_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(dtype=np.uint16, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(dtype=np.uint32, flags="C_CONTIGUOUS")
_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_i64, _i32, _f32, _f64 = C.c_int64, C.c_int, C.c_float, C.c_double


def _sig(name, restype, *argtypes):
    fn = getattr(_lib, name)
    fn.restype = restype
    fn.argtypes = list(argtypes)
    return fn


_h2f = _sig("kvqo_h2f", C.c_float, C.c_uint16)
_f2h = _sig("kvqo_f2h", C.c_uint16, C.c_float)
_codes_bytes = _sig("kvqo_codes_bytes", _i64, _i32, _i32, _i64)
_k_get = _sig("kvqo_k_get", C.c_uint, _u8p, _i32, _i64, _i64, _i32)
_v_get = _sig("kvqo_v_get", C.c_uint, _u8p, _i32, _i64, _i64, _i32)
_pack_k = _sig("kvqo_pack_k", None, _u8p, _i32, _i32, _i64, _i64, _i64, _u8p)
_unpack_k = _sig("kvqo_unpack_k", None, _u8p, _i32, _i32, _i64, _i64, _i64, _u8p)
_pack_v = _sig("kvqo_pack_v", None, _u8p, _i32, _i32, _i64, _i64, _i64, _u8p)
_unpack_v = _sig("kvqo_unpack_v", None, _u8p, _i32, _i32, _i64, _i64, _i64, _u8p)
_nearest = _sig("kvqo_nearest", _i32, _f32p, _i32, _f32)
_store_lut = _sig("kvqo_store_lut", None, _f32p, _i32, _f32p)
_quantize_k = _sig("kvqo_quantize_k", _i64, _u16p, _i64, _i32, _i32, _f32p, _u16p, _u16p, _u16p, _u16p,
                   _u8p, _u32p, _u16p, _u16p, _i64)
_quantize_v = _sig("kvqo_quantize_v", _i64, _u16p, _i64, _i32, _i32, _f32p, _i32, _u16p, _u8p, _u32p,
                   _u16p, _u16p, _i64)
_reconstruct_k = _sig("kvqo_reconstruct_k", None, _u8p, _i32, _i32, _i64, _f32p, _u16p, _u16p, _u32p,
                      _u16p, _u16p, _i64, _i64, _f64p)
_reconstruct_v = _sig("kvqo_reconstruct_v", None, _u8p, _i32, _i32, _i64, _f32p, _u16p, _u32p, _u16p,
                      _u16p, _i64, _i64, _f64p)
_rope = _sig("kvqo_rope", None, _f64p, _i32, _i64, _f64, _f64p)
_qk = _sig("kvqo_qk", None, _u8p, _i32, _i32, _i32, _i64, _i64, _f32p, _u16p, _u16p, _u32p, _u16p, _u16p,
           _f32p, _f32, _f64, _f32p, _i64, _i64, _u16p)
_softmax = _sig("kvqo_softmax", None, _f32p, _i32, _i64, _i64, _f32p, _i64)
_pv = _sig("kvqo_pv", None, _u8p, _i32, _i32, _i32, _i64, _i64, _f32p, _u16p, _u32p, _u16p, _u16p,
           _f32p, _i64, _f32p, _i64, _u16p)
_set_threads = _sig("kvqo_set_threads", None, _i32)
_get_max_threads = _sig("kvqo_get_max_threads", _i32)

HEAD_DIM = 128


def h2f(bits: int) -> float:
    return float(_h2f(int(bits)))


def f2h(x: float) -> int:
    return int(_f2h(float(np.float32(x))))


def set_threads(n: int) -> None:
    _set_threads(int(n))


def max_threads() -> int:
    return int(_get_max_threads())


def codes_bytes(bits: int, n_kv_heads: int, cap: int) -> int:
    return int(_codes_bytes(bits, n_kv_heads, cap))


def _as_bits(x) -> np.ndarray:
    """fp16 array (or uint16 bit patterns) -> contiguous uint16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.float16:
        return np.ascontiguousarray(x).view(np.uint16)
    assert x.dtype == np.uint16
    return np.ascontiguousarray(x)


def store_lut(lut) -> np.ndarray:
    """The signpost table as a cache stores it: every entry rounded to the nearest fp16 number."""
    lut = np.ascontiguousarray(lut, dtype=np.float32)
    out = np.empty_like(lut)
    _store_lut(lut, lut.size, out)
    return out


def nearest(lut: np.ndarray, xn: float) -> int:
    lut = np.ascontiguousarray(lut, dtype=np.float32)
    return int(_nearest(lut, lut.size, float(np.float32(xn))))


def rope(x: np.ndarray, n: int, base: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    _rope(x, x.size, int(n), float(base), y)
    return y


def quantize_k(x, bits, lut, s, z, lo, hi):
    """x: fp16 [T][D].  Returns codes u8 [T][D], cnt u32 [T], idx u16 [nnz], val u16 [nnz]."""
    xb = _as_bits(x)
    T, D = xb.shape
    codes = np.zeros((T, D), dtype=np.uint8)
    cnt = np.zeros(T, dtype=np.uint32)
    idx = np.zeros(T * D, dtype=np.uint16)
    val = np.zeros(T * D, dtype=np.uint16)
    total = _quantize_k(xb, T, D, bits, np.ascontiguousarray(lut, dtype=np.float32), _as_bits(s), _as_bits(z),
                        _as_bits(lo), _as_bits(hi), codes, cnt, idx, val, T * D)
    return codes, cnt, idx[:total].copy(), val[:total].copy()


def quantize_v(x, bits, lut, k_side):
    """x: fp16 [T][D].  Returns sz u16 [T][2], codes, cnt, idx, val."""
    xb = _as_bits(x)
    T, D = xb.shape
    sz = np.zeros((T, 2), dtype=np.uint16)
    codes = np.zeros((T, D), dtype=np.uint8)
    cnt = np.zeros(T, dtype=np.uint32)
    idx = np.zeros(max(1, T * 2 * k_side), dtype=np.uint16)
    val = np.zeros(max(1, T * 2 * k_side), dtype=np.uint16)
    total = _quantize_v(xb, T, D, bits, np.ascontiguousarray(lut, dtype=np.float32), k_side, sz, codes, cnt,
                        idx, val, idx.size)
    if total < 0:
        raise ValueError("2*k_side must be smaller than D")
    return sz, codes, cnt, idx[:total].copy(), val[:total].copy()


def softmax(scores: np.ndarray) -> np.ndarray:
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    H, L = scores.shape
    probs = np.empty_like(scores)
    _softmax(scores, H, L, L, probs, L)
    return probs


class OracleCache:
    """One layer's quantized KV cache held in numpy arrays, driven by the C oracle."""

    def __init__(self, bits, n_kv_heads, n_q_heads, cap_tokens, k_side_v, rope_base,
                 lut_k, lut_v, s_k, z_k, lo_k, hi_k, cap_nnz_k=None, cap_nnz_v=None, n_sink=0):
        assert cap_tokens % 128 == 0
        self.bits, self.H, self.Hq, self.cap = bits, n_kv_heads, n_q_heads, cap_tokens
        self.D = n_kv_heads * HEAD_DIM
        self.k_side_v = k_side_v
        self.rope_base = float(rope_base)
        # the cache stores fp16 signposts (see kvqo_store_lut); everything below uses the stored values
        self.lut_k = store_lut(lut_k)
        self.lut_v = store_lut(lut_v)
        self.s_k, self.z_k, self.lo_k, self.hi_k = (_as_bits(a).copy() for a in (s_k, z_k, lo_k, hi_k))
        nbytes = codes_bytes(bits, n_kv_heads, cap_tokens)
        self.k_codes = np.zeros(nbytes, dtype=np.uint8)
        self.v_codes = np.zeros(nbytes, dtype=np.uint8)
        self.v_sz = np.zeros((cap_tokens, 2), dtype=np.uint16)
        self.cap_nnz_k = int(cap_nnz_k if cap_nnz_k is not None else cap_tokens * self.D)
        self.cap_nnz_v = int(cap_nnz_v if cap_nnz_v is not None else max(1, cap_tokens * 2 * k_side_v))
        self.k_ptr = np.zeros(cap_tokens + 1, dtype=np.uint32)
        self.v_ptr = np.zeros(cap_tokens + 1, dtype=np.uint32)
        self.k_idx = np.zeros(self.cap_nnz_k, dtype=np.uint16)
        self.k_val = np.zeros(self.cap_nnz_k, dtype=np.uint16)
        self.v_idx = np.zeros(self.cap_nnz_v, dtype=np.uint16)
        self.v_val = np.zeros(self.cap_nnz_v, dtype=np.uint16)
        self.n_k = 0
        self.n_v = 0
        # attention-sink tokens (paper Sec. 3.5): the first n_sink tokens are also kept in fp16 and the
        # mat-vecs use those values instead of the quantized ones
        self.n_sink = int(n_sink)
        self.sink_k = np.zeros((max(1, self.n_sink), self.D), dtype=np.uint16)
        self.sink_v = np.zeros((max(1, self.n_sink), self.D), dtype=np.uint16)

    def _append_sparse(self, ptr, idxa, vala, n0, cnt, idx, val):
        for t, c in enumerate(cnt):
            ptr[n0 + t + 1] = ptr[n0 + t] + c
        base = int(ptr[n0])
        idxa[base:base + idx.size] = idx
        vala[base:base + val.size] = val

    def append_k(self, x):
        T = x.shape[0]
        assert self.n_k + T <= self.cap
        codes, cnt, idx, val = quantize_k(x, self.bits, self.lut_k, self.s_k, self.z_k, self.lo_k, self.hi_k)
        _pack_k(self.k_codes, self.bits, self.H, self.cap, self.n_k, T, codes)
        self._append_sparse(self.k_ptr, self.k_idx, self.k_val, self.n_k, cnt, idx, val)
        for t in range(T):
            if self.n_k + t < self.n_sink:
                self.sink_k[self.n_k + t] = _as_bits(x)[t]
        self.n_k += T
        return codes

    def append_v(self, x):
        T = x.shape[0]
        assert self.n_v + T <= self.cap
        sz, codes, cnt, idx, val = quantize_v(x, self.bits, self.lut_v, self.k_side_v)
        _pack_v(self.v_codes, self.bits, self.H, self.cap, self.n_v, T, codes)
        self.v_sz[self.n_v:self.n_v + T] = sz
        self._append_sparse(self.v_ptr, self.v_idx, self.v_val, self.n_v, cnt, idx, val)
        for t in range(T):
            if self.n_v + t < self.n_sink:
                self.sink_v[self.n_v + t] = _as_bits(x)[t]
        self.n_v += T
        return codes

    def unpack_k(self, n0, T):
        codes = np.zeros((T, self.D), dtype=np.uint8)
        _unpack_k(self.k_codes, self.bits, self.H, self.cap, n0, T, codes)
        return codes

    def unpack_v(self, n0, T):
        codes = np.zeros((T, self.D), dtype=np.uint8)
        _unpack_v(self.v_codes, self.bits, self.H, self.cap, n0, T, codes)
        return codes

    def reconstruct_k(self, n0, T):
        out = np.zeros((T, self.D), dtype=np.float64)
        _reconstruct_k(self.k_codes, self.bits, self.H, self.cap, self.lut_k, self.s_k, self.z_k, self.k_ptr,
                       self.k_idx, self.k_val, n0, T, out)
        return out

    def reconstruct_v(self, n0, T):
        out = np.zeros((T, self.D), dtype=np.float64)
        _reconstruct_v(self.v_codes, self.bits, self.H, self.cap, self.lut_v, self.v_sz, self.v_ptr,
                       self.v_idx, self.v_val, n0, T, out)
        return out

    def qk(self, q, scale, L=None):
        L = self.n_k if L is None else L
        q = np.ascontiguousarray(q, dtype=np.float32)
        scores = np.zeros((self.Hq, L), dtype=np.float32)
        _qk(self.k_codes, self.bits, self.H, self.Hq, self.cap, L, self.lut_k, self.s_k, self.z_k, self.k_ptr,
            self.k_idx, self.k_val, q, float(scale), self.rope_base, scores, L, self.n_sink, self.sink_k)
        return scores

    def pv(self, probs, L=None):
        L = self.n_v if L is None else L
        probs = np.ascontiguousarray(probs, dtype=np.float32)
        out = np.zeros((self.Hq, HEAD_DIM), dtype=np.float32)
        _pv(self.v_codes, self.bits, self.H, self.Hq, self.cap, L, self.lut_v, self.v_sz, self.v_ptr,
            self.v_idx, self.v_val, probs, probs.shape[1], out, self.n_sink, self.sink_v)
        return out
