"""CPU oracle for the FP8 linear path (test infrastructure, not product code).

Thin ctypes wrapper over ``llmq_oracle.c`` (plain C, fp64 where it matters).
Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the GPU library never does.

Arrays are numpy: BF16 tensors travel as ``uint16`` bit patterns, FP8 tensors
as ``uint8`` codes.  Formats: ``E4M3 = 0``, ``E5M2 = 1``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

E4M3 = 0
E5M2 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "llmq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no FMA contraction, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-fno-fast-math", "-Wall", "-Wextra", _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    u8p, u16p, f64p, i64p = (c.POINTER(c.c_uint8), c.POINTER(c.c_uint16),
                             c.POINTER(c.c_double), c.POINTER(c.c_int64))
    lib.oracle_fp8_max.restype = c.c_double
    lib.oracle_fp8_max.argtypes = [c.c_int]
    lib.oracle_bf16_to_f32.restype = c.c_float
    lib.oracle_bf16_to_f32.argtypes = [c.c_uint16]
    lib.oracle_f64_to_bf16.restype = c.c_uint16
    lib.oracle_f64_to_bf16.argtypes = [c.c_double]
    lib.oracle_fp8_decode.restype = c.c_double
    lib.oracle_fp8_decode.argtypes = [c.c_uint8, c.c_int]
    lib.oracle_fp8_encode.restype = c.c_uint8
    lib.oracle_fp8_encode.argtypes = [c.c_float, c.c_int]
    lib.oracle_fp8_encode_array.restype = None
    lib.oracle_fp8_encode_array.argtypes = [c.POINTER(c.c_float), c.c_size_t, c.c_int, u8p]
    lib.oracle_amax_bf16.restype = c.c_float
    lib.oracle_amax_bf16.argtypes = [u16p, c.c_size_t]
    lib.oracle_scale.restype = c.c_float
    lib.oracle_scale.argtypes = [c.c_float, c.c_int]
    lib.oracle_quantize.restype = None
    lib.oracle_quantize.argtypes = [u16p, c.c_int64, c.c_int64, c.c_float, c.c_int, u8p, u8p]
    lib.oracle_gemm_tn.restype = None
    lib.oracle_gemm_tn.argtypes = [u8p, c.c_int, u8p, c.c_int, c.c_int64, c.c_int64, c.c_int64,
                                   c.c_float, c.c_float, f64p, f64p]
    lib.oracle_gemm_tn_sampled.restype = None
    lib.oracle_gemm_tn_sampled.argtypes = [u8p, c.c_int, u8p, c.c_int, c.c_int64, c.c_int64,
                                           c.c_int64, c.c_float, c.c_float, i64p, i64p,
                                           c.c_int64, f64p, f64p]
    lib.oracle_sigmoid_exact.restype = c.c_double
    lib.oracle_sigmoid_exact.argtypes = [c.c_double]
    lib.oracle_sigmoid_f32.restype = c.c_float
    lib.oracle_sigmoid_f32.argtypes = [c.c_float]
    lib.oracle_swiglu_fwd.restype = None
    lib.oracle_swiglu_fwd.argtypes = [u16p, c.c_int64, c.c_int64, u16p]
    lib.oracle_swiglu_fwd_exact.restype = None
    lib.oracle_swiglu_fwd_exact.argtypes = [u16p, c.c_int64, c.c_int64, f64p]
    lib.oracle_swiglu_bwd.restype = None
    lib.oracle_swiglu_bwd.argtypes = [u16p, u16p, c.c_int64, c.c_int64, u16p]
    lib.oracle_swiglu_bwd_exact.restype = None
    lib.oracle_swiglu_bwd_exact.argtypes = [u16p, u16p, c.c_int64, c.c_int64, f64p]
    f32p = c.POINTER(c.c_float)
    lib.oracle_residual_add.restype = None
    lib.oracle_residual_add.argtypes = [u16p, u16p, c.c_size_t, u16p]
    lib.oracle_rms_rstd.restype = None
    lib.oracle_rms_rstd.argtypes = [u16p, c.c_int64, c.c_int64, c.c_double, f64p]
    lib.oracle_rmsnorm_exact.restype = None
    lib.oracle_rmsnorm_exact.argtypes = [u16p, u16p, c.c_int64, c.c_int64, c.c_double, f64p]
    lib.oracle_rmsnorm_apply.restype = None
    lib.oracle_rmsnorm_apply.argtypes = [u16p, u16p, f32p, c.c_int64, c.c_int64, u16p]
    lib.oracle_gemm_bf16_tn.restype = None
    lib.oracle_gemm_bf16_tn.argtypes = [u16p, u16p, c.c_int64, c.c_int64, c.c_int64, f64p, f64p]
    lib.oracle_gemm_bf16_tn_sampled.restype = None
    lib.oracle_gemm_bf16_tn_sampled.argtypes = [u16p, u16p, c.c_int64, i64p, i64p, c.c_int64, f64p, f64p]
    lib.oracle_num_threads.restype = c.c_int
    lib.oracle_num_threads.argtypes = []
    _lib = lib
    return lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _as(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, a.dtype))
    return a


def fp8_max(fmt: int) -> float:
    return float(_load().oracle_fp8_max(fmt))


def bf16_to_f32(bits: int) -> float:
    return float(_load().oracle_bf16_to_f32(int(bits)))


def f64_to_bf16(v: float) -> int:
    return int(_load().oracle_f64_to_bf16(float(v)))


def fp8_decode(code: int, fmt: int) -> float:
    return float(_load().oracle_fp8_decode(int(code), fmt))


def fp8_encode(p: float, fmt: int) -> int:
    """Encode one binary32 value (the argument is rounded to binary32 by ctypes)."""
    return int(_load().oracle_fp8_encode(ctypes.c_float(p), fmt))


def fp8_encode_array(p: np.ndarray, fmt: int) -> np.ndarray:
    p = _as(p, np.float32)
    out = np.empty(p.shape, np.uint8)
    _load().oracle_fp8_encode_array(_ptr(p, ctypes.c_float), p.size, fmt, _ptr(out, ctypes.c_uint8))
    return out


def decode_table(fmt: int) -> np.ndarray:
    return np.array([fp8_decode(c, fmt) for c in range(256)], dtype=np.float64)


def amax_bf16(x_bits: np.ndarray) -> np.float32:
    x = _as(x_bits, np.uint16)
    return np.float32(_load().oracle_amax_bf16(_ptr(x, ctypes.c_uint16), x.size))


def scale(amax, fmt: int) -> np.float32:
    return np.float32(_load().oracle_scale(ctypes.c_float(float(amax)), fmt))


def quantize(x_bits: np.ndarray, scale_, fmt: int, transpose: bool = True):
    """Return (q[rows, cols], qt[cols, rows] or None) as uint8 codes."""
    x = _as(x_bits, np.uint16)
    rows, cols = x.shape
    q = np.empty((rows, cols), np.uint8)
    qt = np.empty((cols, rows), np.uint8) if transpose else None
    _load().oracle_quantize(_ptr(x, ctypes.c_uint16), rows, cols, ctypes.c_float(float(scale_)),
                            fmt, _ptr(q, ctypes.c_uint8),
                            _ptr(qt, ctypes.c_uint8) if transpose else None)
    return q, qt


def gemm_tn(A: np.ndarray, fmtA: int, B: np.ndarray, fmtB: int, sA, sB):
    """y[r,c] = sum_t dec(A[r,t]) dec(B[c,t]) / (sA sB) and the matching sum of |products|."""
    A = _as(A, np.uint8)
    B = _as(B, np.uint8)
    R, T = A.shape
    C, T2 = B.shape
    if T != T2:
        raise ValueError("contraction lengths differ")
    y = np.empty((R, C), np.float64)
    S = np.empty((R, C), np.float64)
    _load().oracle_gemm_tn(_ptr(A, ctypes.c_uint8), fmtA, _ptr(B, ctypes.c_uint8), fmtB, R, C, T,
                           ctypes.c_float(float(sA)), ctypes.c_float(float(sB)),
                           _ptr(y, ctypes.c_double), _ptr(S, ctypes.c_double))
    return y, S


def gemm_tn_sampled(A, fmtA, B, fmtB, sA, sB, rr, cc):
    A = _as(A, np.uint8)
    B = _as(B, np.uint8)
    R, T = A.shape
    C, T2 = B.shape
    if T != T2:
        raise ValueError("contraction lengths differ")
    rr = np.ascontiguousarray(rr, dtype=np.int64)
    cc = np.ascontiguousarray(cc, dtype=np.int64)
    if rr.shape != cc.shape or rr.ndim != 1:
        raise ValueError("index lists must be 1-D and equally long")
    if rr.size and (rr.min() < 0 or rr.max() >= R or cc.min() < 0 or cc.max() >= C):
        raise IndexError("sample index out of range")
    y = np.empty(rr.shape, np.float64)
    S = np.empty(rr.shape, np.float64)
    _load().oracle_gemm_tn_sampled(_ptr(A, ctypes.c_uint8), fmtA, _ptr(B, ctypes.c_uint8), fmtB,
                                   R, C, T, ctypes.c_float(float(sA)), ctypes.c_float(float(sB)),
                                   _ptr(rr, ctypes.c_int64), _ptr(cc, ctypes.c_int64), rr.size,
                                   _ptr(y, ctypes.c_double), _ptr(S, ctypes.c_double))
    return y, S


def sigmoid_exact(g: float) -> float:
    return float(_load().oracle_sigmoid_exact(float(g)))


def sigmoid_f32(g) -> np.float32:
    """The binary32 evaluation of the logistic function that the SwiGLU oracle uses."""
    return np.float32(_load().oracle_sigmoid_f32(ctypes.c_float(float(g))))


def _gu_shape(gu_bits):
    gu = _as(gu_bits, np.uint16)
    if gu.ndim != 2 or gu.shape[1] % 2:
        raise ValueError("GU must be [M, 2I]")
    return gu, gu.shape[0], gu.shape[1] // 2


def swiglu_fwd(gu_bits: np.ndarray) -> np.ndarray:
    """h[M, I] as BF16 bit patterns from GU[M, 2I] (gate columns first, then up)."""
    gu, M, I = _gu_shape(gu_bits)
    h = np.empty((M, I), np.uint16)
    _load().oracle_swiglu_fwd(_ptr(gu, ctypes.c_uint16), M, I, _ptr(h, ctypes.c_uint16))
    return h


def swiglu_fwd_exact(gu_bits: np.ndarray) -> np.ndarray:
    gu, M, I = _gu_shape(gu_bits)
    h = np.empty((M, I), np.float64)
    _load().oracle_swiglu_fwd_exact(_ptr(gu, ctypes.c_uint16), M, I, _ptr(h, ctypes.c_double))
    return h


def swiglu_bwd(dh_bits: np.ndarray, gu_bits: np.ndarray) -> np.ndarray:
    """dGU[M, 2I] as BF16 bit patterns from dh[M, I] and GU[M, 2I]."""
    gu, M, I = _gu_shape(gu_bits)
    dh = _as(dh_bits, np.uint16)
    if dh.shape != (M, I):
        raise ValueError("dh must be [M, I]")
    out = np.empty((M, 2 * I), np.uint16)
    _load().oracle_swiglu_bwd(_ptr(dh, ctypes.c_uint16), _ptr(gu, ctypes.c_uint16), M, I,
                              _ptr(out, ctypes.c_uint16))
    return out


def swiglu_bwd_exact(dh_bits: np.ndarray, gu_bits: np.ndarray) -> np.ndarray:
    gu, M, I = _gu_shape(gu_bits)
    dh = _as(dh_bits, np.uint16)
    if dh.shape != (M, I):
        raise ValueError("dh must be [M, I]")
    out = np.empty((M, 2 * I), np.float64)
    _load().oracle_swiglu_bwd_exact(_ptr(dh, ctypes.c_uint16), _ptr(gu, ctypes.c_uint16), M, I,
                                    _ptr(out, ctypes.c_double))
    return out


def residual_add(res_bits: np.ndarray, x_bits: np.ndarray) -> np.ndarray:
    """bf16(res + x) element-wise, as BF16 bit patterns."""
    r, x = _as(res_bits, np.uint16), _as(x_bits, np.uint16)
    if r.shape != x.shape:
        raise ValueError("shapes differ")
    out = np.empty(r.shape, np.uint16)
    _load().oracle_residual_add(_ptr(r, ctypes.c_uint16), _ptr(x, ctypes.c_uint16), r.size, _ptr(out, ctypes.c_uint16))
    return out


def rms_rstd(res_bits: np.ndarray, eps: float) -> np.ndarray:
    """1 / sqrt(mean_c res^2 + eps) per row, binary64."""
    r = _as(res_bits, np.uint16)
    M, C = r.shape
    out = np.empty((M,), np.float64)
    _load().oracle_rms_rstd(_ptr(r, ctypes.c_uint16), M, C, float(eps), _ptr(out, ctypes.c_double))
    return out


def rmsnorm_exact(res_bits: np.ndarray, w_bits: np.ndarray, eps: float) -> np.ndarray:
    r, w = _as(res_bits, np.uint16), _as(w_bits, np.uint16)
    M, C = r.shape
    if w.shape != (C,):
        raise ValueError("w must be [C]")
    y = np.empty((M, C), np.float64)
    _load().oracle_rmsnorm_exact(_ptr(r, ctypes.c_uint16), _ptr(w, ctypes.c_uint16), M, C, float(eps),
                                 _ptr(y, ctypes.c_double))
    return y


def rmsnorm_apply(res_bits: np.ndarray, w_bits: np.ndarray, rstd: np.ndarray) -> np.ndarray:
    """y = bf16((res * rstd[m]) * w[c]) in binary32, as BF16 bit patterns."""
    r, w, s = _as(res_bits, np.uint16), _as(w_bits, np.uint16), _as(rstd, np.float32)
    M, C = r.shape
    if w.shape != (C,) or s.shape != (M,):
        raise ValueError("w must be [C] and rstd [M]")
    y = np.empty((M, C), np.uint16)
    _load().oracle_rmsnorm_apply(_ptr(r, ctypes.c_uint16), _ptr(w, ctypes.c_uint16), _ptr(s, ctypes.c_float),
                                 M, C, _ptr(y, ctypes.c_uint16))
    return y


def gemm_bf16_tn(A_bits: np.ndarray, B_bits: np.ndarray):
    """y[r,c] = sum_t A[r,t] B[c,t] on BF16 bit patterns, binary64, with the matching sum of |products|."""
    A, B = _as(A_bits, np.uint16), _as(B_bits, np.uint16)
    R, T = A.shape
    C, T2 = B.shape
    if T != T2:
        raise ValueError("contraction lengths differ")
    y = np.empty((R, C), np.float64)
    S = np.empty((R, C), np.float64)
    _load().oracle_gemm_bf16_tn(_ptr(A, ctypes.c_uint16), _ptr(B, ctypes.c_uint16), R, C, T,
                                _ptr(y, ctypes.c_double), _ptr(S, ctypes.c_double))
    return y, S


def gemm_bf16_tn_sampled(A_bits, B_bits, rr, cc):
    A, B = _as(A_bits, np.uint16), _as(B_bits, np.uint16)
    R, T = A.shape
    C, T2 = B.shape
    if T != T2:
        raise ValueError("contraction lengths differ")
    rr = np.ascontiguousarray(rr, dtype=np.int64)
    cc = np.ascontiguousarray(cc, dtype=np.int64)
    if rr.shape != cc.shape or rr.ndim != 1:
        raise ValueError("index lists must be 1-D and equally long")
    if rr.size and (rr.min() < 0 or rr.max() >= R or cc.min() < 0 or cc.max() >= C):
        raise IndexError("sample index out of range")
    y = np.empty(rr.shape, np.float64)
    S = np.empty(rr.shape, np.float64)
    _load().oracle_gemm_bf16_tn_sampled(_ptr(A, ctypes.c_uint16), _ptr(B, ctypes.c_uint16), T,
                                        _ptr(rr, ctypes.c_int64), _ptr(cc, ctypes.c_int64), rr.size,
                                        _ptr(y, ctypes.c_double), _ptr(S, ctypes.c_double))
    return y, S


def num_threads() -> int:
    return int(_load().oracle_num_threads())
