"""ctypes front end of the weight-only INT4 oracle (``w4a16_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  It marshals numpy
arrays into the C functions and adds no arithmetic of its own.  binary16
tensors are numpy ``float16`` arrays; the C side sees their bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "w4a16_oracle.c")
_LIB = os.path.join(_HERE, "libw4a16_oracle.so")

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
          "-Wall", "-Wextra"]

GROUP = 128  # group size of the paper's LLM setting (Sec. 4.4)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, no intrinsics, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.w4o_f16_to_f32.restype = C.c_float
        _lib.w4o_f16_to_f32.argtypes = [C.c_uint16]
        _lib.w4o_f32_to_f16.restype = C.c_uint16
        _lib.w4o_f32_to_f16.argtypes = [C.c_float]
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _h(a):
    """float16 array -> contiguous view of its bit patterns."""
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16
    return a.view(np.uint16)


def f16_to_f32(bits: int) -> np.float32:
    return np.float32(lib().w4o_f16_to_f32(C.c_uint16(int(bits))))


def f32_to_f16(x) -> int:
    return int(lib().w4o_f32_to_f16(C.c_float(float(np.float32(x)))))


def quantize_groupwise(w, group: int = GROUP):
    """Eq. 1-2 at 4 bits per group -> (codes uint8 [n,k], scales float16 [n,k/group],
    zeros uint8 [n,k/group])."""
    w = _f32(w)
    n, k = w.shape
    assert k % group == 0
    codes = np.empty((n, k), dtype=np.uint8)
    scales = np.empty((n, k // group), dtype=np.uint16)
    zeros = np.empty((n, k // group), dtype=np.uint8)
    lib().w4o_quantize_groupwise(_p(w, C.c_float), C.c_int64(n), C.c_int64(k), C.c_int64(k),
                                 C.c_int64(group), _p(codes, C.c_uint8), _p(scales, C.c_uint16),
                                 _p(zeros, C.c_uint8))
    return codes, scales.view(np.float16), zeros


def dequant(codes, scales, zeros, group: int = GROUP):
    """Wd = RN16(s * (c - z)) as float32 holding exact binary16 values."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    sb = _h(scales)
    n, k = codes.shape
    wd = np.empty((n, k), dtype=np.float32)
    lib().w4o_dequant(_p(codes, C.c_uint8), _p(sb, C.c_uint16), _p(zeros, C.c_uint8),
                      C.c_int64(n), C.c_int64(k), C.c_int64(group), _p(wd, C.c_float))
    return wd


def product(x16, wd, rows=None):
    """Exact (fp64) layer product and the sum of |terms| -> (acc, mag), each [rows, n]."""
    xb = _h(x16)
    wd = _f32(wd)
    m, k = xb.shape
    n = wd.shape[0]
    assert wd.shape[1] == k
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        cnt = rows.size
    else:
        cnt = m
    acc = np.empty((cnt, n), dtype=np.float64)
    mag = np.empty((cnt, n), dtype=np.float64)
    lib().w4o_product(_p(xb, C.c_uint16), _p(wd, C.c_float), C.c_int64(m), C.c_int64(n),
                      C.c_int64(k), _p(rows, C.c_int64), C.c_int64(cnt), _p(acc, C.c_double),
                      _p(mag, C.c_double))
    return acc, mag


def unfolded(acc, bias, alpha, beta):
    """alpha * (acc + b) + beta in fp64 (Sec. 3.3 applied to the layer output)."""
    acc = _f64(acc)
    rows, n = acc.shape
    out = np.empty_like(acc)
    bias, alpha, beta = _f32(bias), _f32(alpha), _f32(beta)
    lib().w4o_unfolded(_p(acc, C.c_double), C.c_int64(rows), C.c_int64(n), _p(bias, C.c_float),
                       _p(alpha, C.c_float), _p(beta, C.c_float), _p(out, C.c_double))
    return out


def fold(alpha, beta, bias, n):
    """-> (mult, fbias) of the folded epilogue."""
    alpha, beta, bias = _f32(alpha), _f32(beta), _f32(bias)
    mult = np.empty(n, dtype=np.float32)
    fbias = np.empty(n, dtype=np.float32)
    lib().w4o_fold(_p(alpha, C.c_float), _p(beta, C.c_float), _p(bias, C.c_float), C.c_int64(n),
                   _p(mult, C.c_float), _p(fbias, C.c_float))
    return mult, fbias


def folded_real(acc, mult, fbias):
    acc = _f64(acc)
    rows, n = acc.shape
    out = np.empty_like(acc)
    mult, fbias = _f32(mult), _f32(fbias)
    lib().w4o_folded_real(_p(acc, C.c_double), C.c_int64(rows), C.c_int64(n), _p(mult, C.c_float),
                          _p(fbias, C.c_float), _p(out, C.c_double))
    return out


def epilogue_f32(acc32, mult, fbias):
    """The engine's fp32 epilogue on an fp32 accumulator -> (out32, out16)."""
    acc32 = _f32(acc32)
    rows, n = acc32.shape
    out32 = np.empty((rows, n), dtype=np.float32)
    out16 = np.empty((rows, n), dtype=np.uint16)
    mult, fbias = _f32(mult), _f32(fbias)
    lib().w4o_epilogue_f32(_p(acc32, C.c_float), C.c_int64(rows), C.c_int64(n),
                           _p(mult, C.c_float), _p(fbias, C.c_float), _p(out32, C.c_float),
                           _p(out16, C.c_uint16))
    return out32, out16.view(np.float16)
