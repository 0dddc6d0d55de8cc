"""ctypes front end of the CPU oracle (``cwac_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  It marshals numpy
arrays into the C functions and adds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cwac_oracle.c")
_LIB = os.path.join(_HERE, "libcwac_oracle.so")

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
          "-Wall", "-Wextra"]


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
    return _lib


def _p(a, ct):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _i8(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int8)


def set_threads(n: int) -> None:
    lib().orc_set_threads(C.c_int(n))


def get_threads() -> int:
    return int(lib().orc_get_threads())


# ---------------------------------------------------------------- quantizers
def range_f32(x):
    x = _f32(x).ravel()
    mn, mx = C.c_float(), C.c_float()
    lib().orc_range_f32(_p(x, C.c_float), C.c_int64(x.size), C.byref(mn), C.byref(mx))
    return np.float32(mn.value), np.float32(mx.value)


def qparams_asym(mn, mx, bits=8):
    """Eq. 2 -> (scale, zero-point of the unsigned code)."""
    s, z = C.c_float(), C.c_int32()
    lib().orc_qparams_asym(C.c_float(float(mn)), C.c_float(float(mx)), C.c_int32(bits),
                           C.byref(s), C.byref(z))
    return np.float32(s.value), int(z.value)


def quantize_asym(x, s, z, bits=8):
    """Eq. 1 -> unsigned codes (int32 array, same shape)."""
    x = _f32(x)
    out = np.empty(x.shape, dtype=np.int32)
    lib().orc_quantize_asym(_p(x, C.c_float), C.c_int64(x.size), C.c_float(float(s)),
                            C.c_int32(int(z)), C.c_int32(bits), _p(out, C.c_int32))
    return out


def quantize_act_i8(x, s, z_signed):
    x = _f32(x)
    out = np.empty(x.shape, dtype=np.int8)
    lib().orc_quantize_act_i8(_p(x, C.c_float), C.c_int64(x.size), C.c_float(float(s)),
                              C.c_int32(int(z_signed)), _p(out, C.c_int8))
    return out


def quantize_act_per_tensor(x):
    """Eq. 2 then Eq. 1 on a whole tensor, signed 8-bit storage.
    Returns (q int8, scale, signed zero-point)."""
    mn, mx = range_f32(x)
    s, z_u = qparams_asym(mn, mx, 8)
    return quantize_act_i8(x, s, z_u - 128), s, z_u - 128


def quantize_rows_sym(x):
    """Per-row symmetric quantizer -> (q int8 [rows,k], scale fp32 [rows])."""
    x = _f32(x)
    rows, k = x.shape
    q = np.empty((rows, k), dtype=np.int8)
    s = np.empty(rows, dtype=np.float32)
    lib().orc_quantize_rows_sym(_p(x, C.c_float), C.c_int64(rows), C.c_int64(k), C.c_int64(k),
                                _p(s, C.c_float), _p(q, C.c_int8), C.c_int64(k))
    return q, s


def quantize_act_bits(x, s, z_signed, bits):
    """Eq. 1 at `bits` bits, code - 2^(bits-1) stored in int8."""
    x = _f32(x)
    out = np.empty(x.shape, dtype=np.int8)
    lib().orc_quantize_act_bits(_p(x, C.c_float), C.c_int64(x.size), C.c_float(float(s)),
                                C.c_int32(int(z_signed)), C.c_int32(int(bits)), _p(out, C.c_int8))
    return out


def quantize_rows_sym_bits(x, bits):
    """Per-row symmetric quantizer at `bits` bits -> (q int8 [rows,k], scale fp32 [rows])."""
    x = _f32(x)
    rows, k = x.shape
    q = np.empty((rows, k), dtype=np.int8)
    s = np.empty(rows, dtype=np.float32)
    lib().orc_quantize_rows_sym_bits(_p(x, C.c_float), C.c_int64(rows), C.c_int64(k),
                                     C.c_int64(k), C.c_int32(int(bits)), _p(s, C.c_float),
                                     _p(q, C.c_int8), C.c_int64(k))
    return q, s


# ---------------------------------------------------------------- integer product
def gemm_i8(xq, wq, rows=None):
    xq, wq = _i8(xq), _i8(wq)
    m, k = xq.shape
    n, k2 = wq.shape
    assert k == k2
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < m)
        cnt = rows.size
    else:
        cnt = m
    acc = np.empty((cnt, n), dtype=np.int32)
    lib().orc_gemm_i8(_p(xq, C.c_int8), _p(wq, C.c_int8), C.c_int64(m), C.c_int64(n),
                      C.c_int64(k), _p(rows, C.c_int64), C.c_int64(cnt), _p(acc, C.c_int32))
    return acc


def conv2d_i8(xq, wq, stride=1, pad=0, zx=0):
    """Integer product of a quantized convolution: x_q [B,H,W,C_in], w_q [C_out,KH,KW,C_in]
    -> acc int32 [B*OH*OW, C_out]; positions outside the image hold the zero-point."""
    xq, wq = _i8(xq), _i8(wq)
    b, h, w, c_in = xq.shape
    c_out, kh, kw, c2 = wq.shape
    assert c2 == c_in
    oh, ow = (h + 2 * pad - kh) // stride + 1, (w + 2 * pad - kw) // stride + 1
    acc = np.empty((b * oh * ow, c_out), dtype=np.int32)
    lib().orc_conv2d_i8(_p(xq, C.c_int8), _p(wq, C.c_int8), C.c_int64(b), C.c_int64(h),
                        C.c_int64(w), C.c_int64(c_in), C.c_int64(c_out), C.c_int64(kh),
                        C.c_int64(kw), C.c_int64(stride), C.c_int64(pad), C.c_int32(int(zx)),
                        _p(acc, C.c_int32))
    return acc


def colsum_i8(wq):
    wq = _i8(wq)
    n, k = wq.shape
    out = np.empty(n, dtype=np.int32)
    lib().orc_colsum_i8(_p(wq, C.c_int8), C.c_int64(n), C.c_int64(k), _p(out, C.c_int32))
    return out


def product_zp_direct(xq, wq, zx, zw):
    xq, wq, zw = _i8(xq), _i8(wq), _i32(zw)
    m, k = xq.shape
    n = wq.shape[0]
    out = np.empty((m, n), dtype=np.int64)
    lib().orc_product_zp_direct(_p(xq, C.c_int8), _p(wq, C.c_int8), C.c_int64(m), C.c_int64(n),
                                C.c_int64(k), C.c_int32(zx), _p(zw, C.c_int32),
                                _p(out, C.c_int64))
    return out


def product_zp_expanded(xq, wq, zx, zw):
    xq, wq, zw = _i8(xq), _i8(wq), _i32(zw)
    m, k = xq.shape
    n = wq.shape[0]
    out = np.empty((m, n), dtype=np.int64)
    lib().orc_product_zp_expanded(_p(xq, C.c_int8), _p(wq, C.c_int8), C.c_int64(m),
                                  C.c_int64(n), C.c_int64(k), C.c_int32(zx), _p(zw, C.c_int32),
                                  _p(out, C.c_int64))
    return out


# ---------------------------------------------------------------- unfolded layer
def deq_scale(sw, sx):
    sw = _f32(sw)
    out = np.empty_like(sw)
    lib().orc_deq_scale(_p(sw, C.c_float), C.c_int64(sw.size), C.c_float(float(sx)),
                        _p(out, C.c_float))
    return out


def dequant_output(acc, colsum, zx, deq, bias=None, sx_row=None):
    acc, colsum, deq = _i32(acc), _i32(colsum), _f32(deq)
    bias, sx_row = _f32(bias), _f32(sx_row)
    rows, n = acc.shape
    y = np.empty((rows, n), dtype=np.float32)
    lib().orc_dequant_output(_p(acc, C.c_int32), C.c_int64(rows), C.c_int64(n),
                             _p(colsum, C.c_int32), C.c_int32(zx), _p(sx_row, C.c_float),
                             _p(deq, C.c_float), _p(bias, C.c_float), _p(y, C.c_float))
    return y


def cwac_apply(yq, alpha, beta):
    yq, alpha, beta = _f32(yq), _f32(alpha), _f32(beta)
    rows, n = yq.shape
    out = np.empty_like(yq)
    lib().orc_cwac_apply(_p(yq, C.c_float), C.c_int64(rows), C.c_int64(n), _p(alpha, C.c_float),
                         _p(beta, C.c_float), _p(out, C.c_float))
    return out


def requant_output(y, sr, zr, qmin=-128, qmax=127):
    y = _f32(y)
    out = np.empty(y.shape, dtype=np.int8)
    lib().orc_requant_output(_p(y, C.c_float), C.c_int64(y.size), C.c_float(float(sr)),
                             C.c_int32(zr), C.c_int32(qmin), C.c_int32(qmax), _p(out, C.c_int8))
    return out


def unfolded_real(acc, colsum, zx, sw, sx, bias, alpha, beta, sr, sx_row=None):
    acc, colsum, sw = _i32(acc), _i32(colsum), _f32(sw)
    bias, alpha, beta, sx_row = _f32(bias), _f32(alpha), _f32(beta), _f32(sx_row)
    rows, n = acc.shape
    u = np.empty((rows, n), dtype=np.float64)
    lib().orc_unfolded_real(_p(acc, C.c_int32), C.c_int64(rows), C.c_int64(n),
                            _p(colsum, C.c_int32), C.c_int32(zx), _p(sx_row, C.c_float),
                            _p(sw, C.c_float), C.c_float(float(sx)), _p(bias, C.c_float),
                            _p(alpha, C.c_float), _p(beta, C.c_float), C.c_float(float(sr)),
                            _p(u, C.c_double))
    return u


# ---------------------------------------------------------------- fit
def channel_moments(yf, yq):
    """-> float64 [5, C]: mean_f, mean_q, var_q, cov_qf, var_f (1/N)."""
    yf, yq = _f32(yf), _f32(yq)
    rows, c = yf.shape
    assert yq.shape == (rows, c)
    mom = np.empty((5, c), dtype=np.float64)
    lib().orc_channel_moments(_p(yf, C.c_float), _p(yq, C.c_float), C.c_int64(rows),
                              C.c_int64(c), C.c_int64(c), C.c_int64(c), _p(mom, C.c_double))
    return mom


def solve(moments, var_eps=1e-12):
    """Eq. 4-5 -> (alpha fp32 [C], beta fp32 [C], n_degenerate)."""
    mom = np.ascontiguousarray(moments, dtype=np.float64)
    c = mom.shape[1]
    alpha = np.empty(c, dtype=np.float32)
    beta = np.empty(c, dtype=np.float32)
    nd = C.c_int32()
    lib().orc_solve(_p(mom, C.c_double), C.c_int64(c), C.c_double(var_eps), _p(alpha, C.c_float),
                    _p(beta, C.c_float), C.byref(nd))
    return alpha, beta, int(nd.value)


def fit(yf, yq, var_eps=1e-12):
    return solve(channel_moments(yf, yq), var_eps)[:2]


# ---------------------------------------------------------------- fold
def fold_int_offset(alpha, beta, sw, bias, colsum, sx, zx, sr):
    """Eq. 10-11 -> (mult fp32 [N], offset int32 [N], n_saturated)."""
    alpha, beta, sw, bias, colsum = _f32(alpha), _f32(beta), _f32(sw), _f32(bias), _i32(colsum)
    n = sw.size
    mult = np.empty(n, dtype=np.float32)
    offset = np.empty(n, dtype=np.int32)
    ns = C.c_int32()
    lib().orc_fold_int_offset(_p(alpha, C.c_float), _p(beta, C.c_float), _p(sw, C.c_float),
                              _p(bias, C.c_float), _p(colsum, C.c_int32), C.c_int64(n),
                              C.c_float(float(sx)), C.c_int32(zx), C.c_float(float(sr)),
                              _p(mult, C.c_float), _p(offset, C.c_int32), C.byref(ns))
    return mult, offset, int(ns.value)


def fold_fp_bias(alpha, beta, sw, bias, colsum, per_token, sx, zx, sr):
    """-> (mult fp32 [N], fbias fp32 [N], offset int32 [N])."""
    alpha, beta, sw, bias, colsum = _f32(alpha), _f32(beta), _f32(sw), _f32(bias), _i32(colsum)
    n = sw.size
    mult = np.empty(n, dtype=np.float32)
    fbias = np.empty(n, dtype=np.float32)
    offset = np.empty(n, dtype=np.int32)
    lib().orc_fold_fp_bias(_p(alpha, C.c_float), _p(beta, C.c_float), _p(sw, C.c_float),
                           _p(bias, C.c_float), _p(colsum, C.c_int32), C.c_int64(n),
                           C.c_int32(int(per_token)), C.c_float(float(sx)), C.c_int32(zx),
                           C.c_float(float(sr)), _p(mult, C.c_float), _p(fbias, C.c_float),
                           _p(offset, C.c_int32))
    return mult, fbias, offset


# ---------------------------------------------------------------- folded forward
def fold_fixed_point(alpha, beta, sw, bias, colsum, sx, zx, sr):
    """Eq. 10-11 with the multiplier as M0 * 2^-shift -> (m0 int32 [N], shift int32 [N],
    offset int32 [N], n_saturated)."""
    sw, colsum = _f32(sw), _i32(colsum)
    alpha, beta, bias = _f32(alpha), _f32(beta), _f32(bias)
    n = sw.shape[0]
    m0 = np.empty(n, dtype=np.int32)
    shift = np.empty(n, dtype=np.int32)
    offset = np.empty(n, dtype=np.int32)
    nsat = C.c_int32()
    lib().orc_fold_fixed_point(_p(alpha, C.c_float), _p(beta, C.c_float), _p(sw, C.c_float),
                               _p(bias, C.c_float), _p(colsum, C.c_int32), C.c_int64(n),
                               C.c_float(sx), C.c_int32(zx), C.c_float(sr), _p(m0, C.c_int32),
                               _p(shift, C.c_int32), _p(offset, C.c_int32), C.byref(nsat))
    return m0, shift, offset, int(nsat.value)


def fixed_point_forward(acc, offset, m0, shift, zr, qmin=-128, qmax=127):
    """Integer-only epilogue of Eq. 10 on integer accumulators -> int8 [rows, N]."""
    acc, offset, m0, shift = _i32(acc), _i32(offset), _i32(m0), _i32(shift)
    rows, n = acc.shape
    out = np.empty((rows, n), dtype=np.int8)
    lib().orc_fixed_point_forward(_p(acc, C.c_int32), C.c_int64(rows), C.c_int64(n),
                                  _p(offset, C.c_int32), _p(m0, C.c_int32), _p(shift, C.c_int32),
                                  C.c_int32(zr), C.c_int32(qmin), C.c_int32(qmax),
                                  _p(out, C.c_int8))
    return out


def folded_forward(acc, offset, mult, zr, fbias=None, sx_row=None, qmin=-128, qmax=127,
                   want_f32=False):
    """Eq. 10 epilogue on integer accumulators -> int8 [rows, N]
    (and the un-rounded fp32 value when want_f32)."""
    acc, offset, mult = _i32(acc), _i32(offset), _f32(mult)
    fbias, sx_row = _f32(fbias), _f32(sx_row)
    rows, n = acc.shape
    out = np.empty((rows, n), dtype=np.int8)
    u = np.empty((rows, n), dtype=np.float32) if want_f32 else None
    lib().orc_folded_forward(_p(acc, C.c_int32), C.c_int64(rows), C.c_int64(n),
                             _p(offset, C.c_int32), _p(sx_row, C.c_float), _p(mult, C.c_float),
                             _p(fbias, C.c_float), C.c_int32(zr), C.c_int32(qmin),
                             C.c_int32(qmax), _p(out, C.c_int8), _p(u, C.c_float))
    return (out, u) if want_f32 else out
