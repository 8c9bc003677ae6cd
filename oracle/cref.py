"""ctypes access to the C oracle (oracle/h1bkv_oracle.c) -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Array arguments are numpy arrays; floating inputs are passed as float32 *values* (an fp16 input is
widened exactly before the call), so one entry point serves both boundary dtypes.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        L.h1bkv_oracle_half_to_float.restype = C.c_float
        L.h1bkv_oracle_half_to_float.argtypes = [C.c_uint16]
        L.h1bkv_oracle_float_to_half.restype = C.c_uint16
        L.h1bkv_oracle_float_to_half.argtypes = [C.c_float]
        L.h1bkv_oracle_max_threads.restype = C.c_int
        for name in ("h1bkv_oracle_sketch", "h1bkv_oracle_quantize", "h1bkv_oracle_dequantize",
                     "h1bkv_oracle_hamming", "h1bkv_oracle_decode_one", "h1bkv_oracle_decode_batch",
                     "h1bkv_oracle_append_batch", "h1bkv_oracle_decode_one_f16v",
                     "h1bkv_oracle_decode_batch_f16v", "h1bkv_oracle_append_batch_f16v",
                     "h1bkv_oracle_prefill_batch", "h1bkv_oracle_decode_one_dtau", "h1bkv_oracle_decode_batch_dtau",
                     "h1bkv_oracle_decode_one_dtau_f16v", "h1bkv_oracle_decode_batch_dtau_f16v"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(np.asarray(a).astype(np.float32))


def max_threads() -> int:
    return int(lib().h1bkv_oracle_max_threads())


def set_threads(n: int) -> None:
    """Threads the oracle's OpenMP loops use from now on (the OpenMP runtime's own call; the oracle is untouched)."""
    lib()
    C.CDLL("libgomp.so.1").omp_set_num_threads(C.c_int(int(n)))


def half_to_float(h: int) -> float:
    return float(lib().h1bkv_oracle_half_to_float(int(h)))


def float_to_half(f: float) -> int:
    return int(lib().h1bkv_oracle_float_to_half(C.c_float(f)))


def sketch(R: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Eq.(2): x [..., d] -> packed sketches [..., b/64] uint64."""
    R = _f32(R)
    b, d = R.shape
    x = _f32(x)
    n = x.size // d
    out = np.zeros((n, b // 64), dtype=np.uint64)
    lib().h1bkv_oracle_sketch(_p(R), C.c_int(b), C.c_int(d), _p(x), C.c_int64(n), _p(out))
    return out.reshape(x.shape[:-1] + (b // 64,))


def quantize(v: np.ndarray, G: int):
    """Eq.(4): v [..., d] -> (codes [..., d/2] u8, scale [..., d/G] u16 fp16 bits, zero [..., d/G] u16)."""
    v = _f32(v)
    d = v.shape[-1]
    n = v.size // d
    codes = np.zeros((n, d // 2), dtype=np.uint8)
    scale = np.zeros((n, d // G), dtype=np.uint16)
    zero = np.zeros((n, d // G), dtype=np.uint16)
    lib().h1bkv_oracle_quantize(_p(v), C.c_int64(n), C.c_int(d), C.c_int(G), _p(codes), _p(scale), _p(zero))
    lead = v.shape[:-1]
    return codes.reshape(lead + (d // 2,)), scale.reshape(lead + (d // G,)), zero.reshape(lead + (d // G,))


def dequantize(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray, G: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scale = np.ascontiguousarray(scale, dtype=np.uint16)
    zero = np.ascontiguousarray(zero, dtype=np.uint16)
    d = codes.shape[-1] * 2
    n = codes.size // (d // 2)
    out = np.zeros((n, d), dtype=np.float64)
    lib().h1bkv_oracle_dequantize(_p(codes), _p(scale), _p(zero), C.c_int64(n), C.c_int(d), C.c_int(G), _p(out))
    return out.reshape(codes.shape[:-1] + (d,))


def hamming(sq: np.ndarray, sk: np.ndarray) -> np.ndarray:
    sq = np.ascontiguousarray(sq, dtype=np.uint64)
    sk = np.ascontiguousarray(sk, dtype=np.uint64)
    T, W = sk.shape
    ham = np.zeros(T, dtype=np.int32)
    lib().h1bkv_oracle_hamming(_p(sq), _p(sk), C.c_int64(T), C.c_int(W), _p(ham))
    return ham


def decode_one(sq, sk, codes, scale, zero, b: int, G: int, tau: float) -> np.ndarray:
    """Eq.(3)+(5) for one (sequence, query head): returns out [d] float32."""
    sq = np.ascontiguousarray(sq, dtype=np.uint64)
    sk = np.ascontiguousarray(sk, dtype=np.uint64)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scale = np.ascontiguousarray(scale, dtype=np.uint16)
    zero = np.ascontiguousarray(zero, dtype=np.uint16)
    T = sk.shape[0]
    d = codes.shape[-1] * 2
    out = np.zeros(d, dtype=np.float32)
    lib().h1bkv_oracle_decode_one(_p(sq), _p(sk), _p(codes), _p(scale), _p(zero), C.c_int64(T), C.c_int(b),
                                  C.c_int(d), C.c_int(G), C.c_double(tau), _p(out))
    return out


def decode_one_dtau(sq, sk, codes, scale, zero, b: int, G: int, tau: float):
    """Eq.(5) and d out / d tau for one (sequence, query head): returns (out [d], dout [d]) float32."""
    sq = np.ascontiguousarray(sq, dtype=np.uint64)
    sk = np.ascontiguousarray(sk, dtype=np.uint64)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scale = np.ascontiguousarray(scale, dtype=np.uint16)
    zero = np.ascontiguousarray(zero, dtype=np.uint16)
    T = sk.shape[0]
    d = codes.shape[-1] * 2
    out = np.zeros(d, dtype=np.float32)
    dout = np.zeros(d, dtype=np.float32)
    lib().h1bkv_oracle_decode_one_dtau(_p(sq), _p(sk), _p(codes), _p(scale), _p(zero), C.c_int64(T), C.c_int(b),
                                       C.c_int(d), C.c_int(G), C.c_double(tau), _p(out), _p(dout))
    return out, dout


def decode_one_f16v(sq, sk, v16, b: int, tau: float) -> np.ndarray:
    """Eq.(3)+(5) with fp16 values (the "1-bit key only" variant): v16 [T][d] fp16 bit patterns -> out [d] float32."""
    sq = np.ascontiguousarray(sq, dtype=np.uint64)
    sk = np.ascontiguousarray(sk, dtype=np.uint64)
    v16 = np.ascontiguousarray(v16, dtype=np.uint16)
    T, d = v16.shape
    out = np.zeros(d, dtype=np.float32)
    lib().h1bkv_oracle_decode_one_f16v(_p(sq), _p(sk), _p(v16), C.c_int64(T), C.c_int(b), C.c_int(d),
                                       C.c_double(tau), _p(out))
    return out


def decode_one_dtau_f16v(sq, sk, v16, b: int, tau: float):
    """Eq.(5) with fp16 values and d out / d tau for one (sequence, query head): returns (out [d], dout [d]) float32."""
    sq = np.ascontiguousarray(sq, dtype=np.uint64)
    sk = np.ascontiguousarray(sk, dtype=np.uint64)
    v16 = np.ascontiguousarray(v16, dtype=np.uint16)
    T, d = v16.shape
    out = np.zeros(d, dtype=np.float32)
    dout = np.zeros(d, dtype=np.float32)
    lib().h1bkv_oracle_decode_one_dtau_f16v(_p(sq), _p(sk), _p(v16), C.c_int64(T), C.c_int(b), C.c_int(d),
                                            C.c_double(tau), _p(out), _p(dout))
    return out, dout


class Cache:
    """Canonical-layout compressed cache on the host: planes [B][H_kv][Tcap][...], filled by the oracle."""

    def __init__(self, R: np.ndarray, B: int, Hkv: int, Tcap: int, G: int, value_bits: int = 4):
        assert value_bits in (4, 16)
        self.R = _f32(R)
        self.b, self.d = self.R.shape
        self.B, self.Hkv, self.Tcap, self.G = B, Hkv, Tcap, G
        self.value_bits = value_bits
        self.W, self.ng = self.b // 64, self.d // G
        self.sketches = np.zeros((B, Hkv, Tcap, self.W), dtype=np.uint64)
        if value_bits == 4:
            self.codes = np.zeros((B, Hkv, Tcap, self.d // 2), dtype=np.uint8)
            self.scale = np.zeros((B, Hkv, Tcap, self.ng), dtype=np.uint16)
            self.zero = np.zeros((B, Hkv, Tcap, self.ng), dtype=np.uint16)
        else:
            self.v16 = np.zeros((B, Hkv, Tcap, self.d), dtype=np.uint16)     # fp16 bit patterns
        self.len = 0

    def append(self, k: np.ndarray, v: np.ndarray) -> None:
        """k, v in boundary layout [B][n_new][H_kv][d]; appended at positions [len, len+n_new)."""
        k, v = _f32(k), _f32(v)
        n_new = k.shape[1]
        assert k.shape == v.shape == (self.B, n_new, self.Hkv, self.d)
        assert self.len + n_new <= self.Tcap
        if self.value_bits == 16:
            lib().h1bkv_oracle_append_batch_f16v(_p(self.R), C.c_int(self.b), C.c_int(self.d), C.c_int(self.B),
                                                 C.c_int(self.Hkv), C.c_int64(self.Tcap), C.c_int64(self.len),
                                                 C.c_int64(n_new), _p(k), _p(v), _p(self.sketches), _p(self.v16))
            self.len += n_new
            return
        lib().h1bkv_oracle_append_batch(_p(self.R), C.c_int(self.b), C.c_int(self.d), C.c_int(self.G),
                                        C.c_int(self.B), C.c_int(self.Hkv), C.c_int64(self.Tcap),
                                        C.c_int64(self.len), C.c_int64(n_new), _p(k), _p(v), _p(self.sketches),
                                        _p(self.codes), _p(self.scale), _p(self.zero))
        self.len += n_new

    def decode(self, q: np.ndarray, tau: float, ctx_len=None) -> np.ndarray:
        """q [B][H_q][d] -> out [B][H_q][d] float32 over the first ctx_len[s] (default: all) tokens."""
        q = _f32(q)
        Hq = q.shape[1]
        lens = np.full(self.B, self.len, dtype=np.int32) if ctx_len is None else np.ascontiguousarray(ctx_len, dtype=np.int32)
        out = np.zeros((self.B, Hq, self.d), dtype=np.float32)
        if self.value_bits == 16:
            lib().h1bkv_oracle_decode_batch_f16v(_p(self.R), C.c_int(self.b), C.c_int(self.d), C.c_int(self.B),
                                                 C.c_int(Hq), C.c_int(self.Hkv), C.c_int64(self.Tcap), _p(lens), _p(q),
                                                 _p(self.sketches), _p(self.v16), C.c_double(tau), _p(out))
            return out
        lib().h1bkv_oracle_decode_batch(_p(self.R), C.c_int(self.b), C.c_int(self.d), C.c_int(self.G),
                                        C.c_int(self.B), C.c_int(Hq), C.c_int(self.Hkv), C.c_int64(self.Tcap),
                                        _p(lens), _p(q), _p(self.sketches), _p(self.codes), _p(self.scale),
                                        _p(self.zero), C.c_double(tau), _p(out))
        return out

    def decode_dtau(self, q: np.ndarray, tau: float, ctx_len=None):
        """q [B][H_q][d] -> (out, d out / d tau), each [B][H_q][d] float32."""
        q = _f32(q)
        Hq = q.shape[1]
        lens = np.full(self.B, self.len, dtype=np.int32) if ctx_len is None else np.ascontiguousarray(ctx_len, dtype=np.int32)
        out = np.zeros((self.B, Hq, self.d), dtype=np.float32)
        dout = np.zeros((self.B, Hq, self.d), dtype=np.float32)
        if self.value_bits == 16:
            lib().h1bkv_oracle_decode_batch_dtau_f16v(_p(self.R), C.c_int(self.b), C.c_int(self.d), C.c_int(self.B),
                                                      C.c_int(Hq), C.c_int(self.Hkv), C.c_int64(self.Tcap), _p(lens), _p(q),
                                                      _p(self.sketches), _p(self.v16), C.c_double(tau), _p(out), _p(dout))
            return out, dout
        lib().h1bkv_oracle_decode_batch_dtau(_p(self.R), C.c_int(self.b), C.c_int(self.d), C.c_int(self.G),
                                             C.c_int(self.B), C.c_int(Hq), C.c_int(self.Hkv), C.c_int64(self.Tcap),
                                             _p(lens), _p(q), _p(self.sketches), _p(self.codes), _p(self.scale),
                                             _p(self.zero), C.c_double(tau), _p(out), _p(dout))
        return out, dout

    def prefill(self, q: np.ndarray, tau: float, ctx_len=None) -> np.ndarray:
        """q [B][n_q][H_q][d]: the last n_q cached positions of every sequence attend causally (each to the tokens up
        to and including its own position) -> out [B][n_q][H_q][d] float32."""
        q = _f32(q)
        n_q, Hq = q.shape[1], q.shape[2]
        lens = np.full(self.B, self.len, dtype=np.int32) if ctx_len is None else np.ascontiguousarray(ctx_len, dtype=np.int32)
        assert (lens >= n_q).all()
        out = np.zeros((self.B, n_q, Hq, self.d), dtype=np.float32)
        if self.value_bits == 16:          # the definition itself: position i is the decode step over its own prefix
            for i in range(n_q):
                out[:, i] = self.decode(q[:, i], tau, ctx_len=lens - n_q + i + 1)
            return out
        lib().h1bkv_oracle_prefill_batch(_p(self.R), C.c_int(self.b), C.c_int(self.d), C.c_int(self.G), C.c_int(self.B),
                                         C.c_int(Hq), C.c_int(self.Hkv), C.c_int64(self.Tcap), _p(lens), C.c_int64(n_q),
                                         _p(q), _p(self.sketches), _p(self.codes), _p(self.scale), _p(self.zero),
                                         C.c_double(tau), _p(out))
        return out
