"""Thin ctypes binding of libcwac_hip.so: one Python function per C entry point,
same names, argument marshalling only.  torch supplies device memory and the
stream handle; every step of the path runs in the library's HIP kernels.  There
is no fallback: a missing library or an error status raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch  # imported first so that the library binds to torch's HIP runtime

_PKG = os.path.dirname(os.path.abspath(__file__))
# CWAC_LIB overrides the library path (development builds); the default is the in-tree build
LIB_PATH = os.environ.get("CWAC_LIB") or os.path.join(_PKG, "libcwac_hip.so")

CWAC_OK = 0
CWAC_EPI_INT_OFFSET, CWAC_EPI_FP_BIAS = 0, 1
CWAC_OUT_INT8, CWAC_OUT_FP32, CWAC_OUT_INT32, CWAC_OUT_FP16 = 0, 1, 2, 3
CWAC_W4_GROUP = 128
# cwac_tuning.kernel / .shape
CWAC_KERNEL_AUTO, CWAC_KERNEL_DIRECT_LDS = 0, 1
CWAC_KERNEL_GENERIC_64, CWAC_KERNEL_GENERIC_128, CWAC_KERNEL_GENERIC_256 = 64, 128, 256
(CWAC_SHAPE_AUTO, CWAC_SHAPE_256_8W, CWAC_SHAPE_256_4W_K128, CWAC_SHAPE_256_4W_K64, CWAC_SHAPE_128_PAIR,
 CWAC_SHAPE_128_128, CWAC_SHAPE_256_PERSIST) = range(7)

EXPORTS = (
    "cwac_status_string", "cwac_range_workspace", "cwac_range_f32", "cwac_qparams_from_range",
    "cwac_quantize_act", "cwac_quantize_rows_sym", "cwac_colsum", "cwac_stats_bytes",
    "cwac_stats_reset", "cwac_calibrate_stats_workspace", "cwac_calibrate_stats", "cwac_solve",
    "cwac_fold", "qlinear_cwac_forward", "cwac_calibrate_fused_workspace",
    "qlinear_cwac_calibrate_fused", "cwac_epilogue_int32", "cwac_apply_unfolded",
    "cwac_mfma_probe", "cwac_mfma_probe_f16", "cwac_hbm_read_probe", "cwac_kloop_probe", "cwac_fold_fixed_point", "qlinear_cwac_forward_fixed_point",
    "cwac_quantize_act_bits", "cwac_quantize_rows_sym_bits",
    "cwac_w4_quantize_groupwise", "cwac_w4_packed_w_bytes", "cwac_w4_pack",
    "cwac_fold_weight_only", "qlinear_w4a16_cwac_forward", "qconv2d_cwac_forward",
    "vit_residual_ln_quant", "vit_gelu_table", "vit_table_lookup", "vit_attention_int8",
    "vit_block_workspace", "vit_block_w8a8_forward", "qlinear_cwac_forward_table",
    "vit_encoder_w8a8_forward", "cwac_calibrate_stats_first",
    "qlinear_cwac_forward_ex", "qlinear_cwac_forward_table_ex", "qconv2d_cwac_forward_ex",
    "qlinear_cwac_calibrate_fused_ex", "qlinear_cwac_forward_fixed_point_ex",
    "qlinear_w4a16_cwac_forward_ex", "cwac_forward_kernel_for",
    "cwac_static_scratch_bytes", "cwac_calibrate_stats_static",
)


class cwac_qparams(C.Structure):
    _fields_ = [("mode", C.c_int32), ("act_per_token", C.c_int32), ("s_x", C.c_float),
                ("z_x", C.c_int32), ("s_r", C.c_float), ("z_r", C.c_int32),
                ("qmin", C.c_int32), ("qmax", C.c_int32)]


class cwac_tuning(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("shape", C.c_int32), ("stats_waves", C.c_int32),
                ("w4_tile", C.c_int32), ("w4_small_waves", C.c_int32), ("persist_workgroups", C.c_int32),
                ("w4_small_depth", C.c_int32), ("persist_loaders", C.c_int32)]


class vit_block_layer(C.Structure):
    _fields_ = [("w_q", C.c_void_p), ("mult", C.c_void_p), ("offset", C.c_void_p), ("s_x", C.c_float),
                ("z_x", C.c_int32), ("s_r", C.c_float), ("z_r", C.c_int32)]


class vit_block_params(C.Structure):
    _fields_ = [("batch", C.c_int32), ("tokens", C.c_int32), ("heads", C.c_int32), ("hidden", C.c_int32),
                ("eps", C.c_float), ("ln1_gamma", C.c_void_p), ("ln1_beta", C.c_void_p),
                ("ln2_gamma", C.c_void_p), ("ln2_beta", C.c_void_p), ("layer", vit_block_layer * 4),
                ("gelu_table", C.c_void_p), ("head_dim", C.c_int32),
                ("attn_bias", C.c_void_p), ("attn_bias_ld", C.c_int64)]


class CwacError(RuntimeError):
    pass


_lib = None


def lib() -> C.CDLL:
    """Loads the HIP library built in-tree (see build.py); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise CwacError(f"{LIB_PATH} is missing: build it with "
                            "`python -m paper_2505_20932_amd.build` (no fallback path exists)")
        l = C.CDLL(LIB_PATH)
        vp, i64, i32, f32, f64, sz = C.c_void_p, C.c_int64, C.c_int32, C.c_float, C.c_double, C.c_size_t
        qpp = C.POINTER(cwac_qparams)
        tup = C.POINTER(cwac_tuning)
        sig = {
            "cwac_status_string": (C.c_char_p, [i32]),
            "cwac_range_workspace": (sz, [i64]),
            "cwac_range_f32": (i32, [vp, i64, vp, vp, sz, vp]),
            "cwac_qparams_from_range": (i32, [f32, f32, i32, C.POINTER(f32), C.POINTER(i32)]),
            "cwac_quantize_act": (i32, [vp, i64, i64, i32, f32, i32, vp, i64, vp]),
            "cwac_quantize_rows_sym": (i32, [vp, i64, i64, i32, vp, vp, i64, vp]),
            "cwac_quantize_act_bits": (i32, [vp, i64, i64, i32, f32, i32, i32, vp, i64, vp]),
            "cwac_quantize_rows_sym_bits": (i32, [vp, i64, i64, i32, i32, vp, vp, i64, vp]),
            "cwac_colsum": (i32, [vp, i64, i32, i32, vp, vp]),
            "cwac_stats_bytes": (sz, [i32]),
            "cwac_stats_reset": (i32, [vp, i32, vp]),
            "cwac_calibrate_stats_workspace": (sz, [i64, i32]),
            "cwac_calibrate_stats": (i32, [vp, i64, vp, i64, i64, i32, vp, vp, sz, vp]),
            "cwac_solve": (i32, [vp, i32, f64, vp, vp, vp, vp, vp]),
            "cwac_fold": (i32, [vp, vp, vp, vp, vp, i32, qpp, vp, vp, vp, vp, vp]),
            "qlinear_cwac_forward": (i32, [vp, i64, vp, i64, i64, i32, i32, qpp, vp, vp, vp, vp,
                                           i32, vp, i64, vp]),
            "cwac_calibrate_fused_workspace": (sz, [i64, i32]),
            "qlinear_cwac_calibrate_fused": (i32, [vp, i64, vp, i64, i64, i32, i32, vp, vp, vp, vp,
                                                   vp, i64, vp, vp, sz, vp]),
            "cwac_epilogue_int32": (i32, [vp, i64, i64, i32, qpp, vp, vp, vp, vp, i32, vp, i64, vp]),
            "cwac_apply_unfolded": (i32, [vp, i64, i64, i32, vp, vp, vp, i64, vp]),
            "cwac_mfma_probe": (i32, [vp, i32, i32, vp, vp]),
            "cwac_mfma_probe_f16": (i32, [vp, i32, i32, vp, vp]),
            "cwac_hbm_read_probe": (i32, [vp, C.c_size_t, i32, vp, vp]),
            "cwac_kloop_probe": (i32, [vp, vp, i32, i32, i32, vp, vp]),
            "cwac_fold_fixed_point": (i32, [vp, vp, vp, vp, vp, i32, qpp, vp, vp, vp, vp, vp]),
            "qlinear_cwac_forward_fixed_point": (i32, [vp, i64, vp, i64, i64, i32, i32, qpp, vp, vp,
                                                       vp, vp, i64, vp]),
            "qconv2d_cwac_forward": (i32, [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, qpp,
                                           vp, vp, vp, i32, vp, i64, vp]),
            "cwac_w4_quantize_groupwise": (i32, [vp, i64, i32, i32, vp, vp, vp, vp]),
            "cwac_w4_packed_w_bytes": (sz, [i32, i32]),
            "cwac_w4_pack": (i32, [vp, vp, vp, i32, i32, vp, vp, vp]),
            "cwac_fold_weight_only": (i32, [vp, vp, vp, i32, vp, vp, vp]),
            "qlinear_w4a16_cwac_forward": (i32, [vp, i64, vp, vp, i64, i32, i32, vp, vp, i32, vp,
                                                 i64, vp]),
            "vit_residual_ln_quant": (i32, [vp, i64, vp, i64, f32, i32, vp, i64, vp, vp, f32, f32, i32,
                                            vp, i64, i64, i32, vp]),
            "vit_gelu_table": (i32, [f32, i32, f32, i32, vp, vp]),
            "vit_table_lookup": (i32, [vp, i64, vp, vp, i64, i64, i32, vp]),
            "vit_attention_int8": (i32, [vp, i64, f32, i32, i32, i32, i32, i32, vp, i64, f32, i32, vp, i64, vp]),
            "vit_block_workspace": (sz, [i32, i32, i32, i32]),
            "qlinear_cwac_forward_table": (i32, [vp, i64, vp, i64, i64, i32, i32, qpp, vp, vp, vp, vp, i64, vp]),
            "vit_block_w8a8_forward": (i32, [C.POINTER(vit_block_params), vp, vp, vp, sz, vp]),
            "vit_encoder_w8a8_forward": (i32, [C.POINTER(vit_block_params), i32, vp, vp, vp, sz, vp]),
        }
        sig["cwac_calibrate_stats_first"] = sig["cwac_calibrate_stats"]
        sig["cwac_static_scratch_bytes"] = (sz, [])
        sig["cwac_calibrate_stats_static"] = (i32, [vp, i64, vp, i64, i64, i32, vp, vp])
        sig["cwac_forward_kernel_for"] = (i32, [i64, i32, i32, i64, i64, i32, tup])
        for name in ("qlinear_cwac_forward", "qlinear_cwac_forward_table", "qconv2d_cwac_forward",
                     "qlinear_cwac_calibrate_fused", "qlinear_cwac_forward_fixed_point",
                     "qlinear_w4a16_cwac_forward"):
            res, args = sig[name]                       # _ex: the same call with a tuning before the stream
            sig[name + "_ex"] = (res, args[:-1] + [tup, vp])
        for name, (res, args) in sig.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(status: int, what: str) -> None:
    if status != CWAC_OK:
        msg = lib().cwac_status_string(status).decode()
        raise CwacError(f"{what}: {msg} ({status})")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda, "device tensor expected"
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _rowmajor(t: torch.Tensor) -> int:
    assert t.dim() == 2 and t.stride(1) == 1, "row-major 2-D tensor expected"
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def make_tuning(kernel=0, shape=0, stats_waves=0, w4_tile=0, w4_small_waves=0,
                persist_workgroups=0, w4_small_depth=0, persist_loaders=0) -> cwac_tuning:
    """Kernel choice override for the ``tuning=`` argument of the forward calls (same results)."""
    return cwac_tuning(int(kernel), int(shape), int(stats_waves), int(w4_tile), int(w4_small_waves),
                       int(persist_workgroups), int(w4_small_depth), int(persist_loaders))


def _tun(tuning: Optional[cwac_tuning]):
    return C.byref(tuning) if tuning is not None else None


def make_qparams(mode=CWAC_EPI_INT_OFFSET, act_per_token=False, s_x=1.0, z_x=0, s_r=1.0, z_r=0,
                 qmin=-128, qmax=127) -> cwac_qparams:
    return cwac_qparams(int(mode), int(bool(act_per_token)), float(s_x), int(z_x), float(s_r),
                        int(z_r), int(qmin), int(qmax))


# --------------------------------------------------------------------------- quantizers
def cwac_range_workspace(count: int) -> int:
    return int(lib().cwac_range_workspace(count))


def cwac_range_f32(x: torch.Tensor, minmax: torch.Tensor, workspace: torch.Tensor, stream=None):
    assert x.dtype == torch.float32 and x.is_contiguous() and minmax.dtype == torch.float32
    _check(lib().cwac_range_f32(_ptr(x), x.numel(), _ptr(minmax), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)),
           "cwac_range_f32")


def cwac_qparams_from_range(mn: float, mx: float, bits: int = 8):
    s, z = C.c_float(), C.c_int32()
    _check(lib().cwac_qparams_from_range(mn, mx, bits, C.byref(s), C.byref(z)),
           "cwac_qparams_from_range")
    return s.value, z.value


def cwac_quantize_act(x: torch.Tensor, s: float, z: int, q: torch.Tensor, stream=None):
    assert x.dtype == torch.float32 and q.dtype == torch.int8 and x.shape == q.shape
    _check(lib().cwac_quantize_act(_ptr(x), _rowmajor(x), x.shape[0], x.shape[1], s, z, _ptr(q),
                                   _rowmajor(q), _stream(stream)), "cwac_quantize_act")


def cwac_quantize_rows_sym(x: torch.Tensor, scale: torch.Tensor, q: torch.Tensor, stream=None):
    assert x.dtype == torch.float32 and q.dtype == torch.int8 and scale.dtype == torch.float32
    assert x.shape == q.shape and scale.numel() == x.shape[0]
    _check(lib().cwac_quantize_rows_sym(_ptr(x), _rowmajor(x), x.shape[0], x.shape[1], _ptr(scale),
                                        _ptr(q), _rowmajor(q), _stream(stream)),
           "cwac_quantize_rows_sym")


def cwac_quantize_act_bits(x: torch.Tensor, s: float, z: int, bits: int, q: torch.Tensor,
                           stream=None):
    assert x.dtype == torch.float32 and q.dtype == torch.int8 and x.shape == q.shape
    _check(lib().cwac_quantize_act_bits(_ptr(x), _rowmajor(x), x.shape[0], x.shape[1], s, z, bits,
                                        _ptr(q), _rowmajor(q), _stream(stream)),
           "cwac_quantize_act_bits")


def cwac_quantize_rows_sym_bits(x: torch.Tensor, bits: int, scale: torch.Tensor, q: torch.Tensor,
                                stream=None):
    assert x.dtype == torch.float32 and q.dtype == torch.int8 and scale.dtype == torch.float32
    assert x.shape == q.shape and scale.numel() == x.shape[0]
    _check(lib().cwac_quantize_rows_sym_bits(_ptr(x), _rowmajor(x), x.shape[0], x.shape[1], bits,
                                             _ptr(scale), _ptr(q), _rowmajor(q), _stream(stream)),
           "cwac_quantize_rows_sym_bits")


def cwac_colsum(w_q: torch.Tensor, colsum: torch.Tensor, stream=None):
    assert w_q.dtype == torch.int8 and colsum.dtype == torch.int32
    _check(lib().cwac_colsum(_ptr(w_q), _rowmajor(w_q), w_q.shape[0], w_q.shape[1], _ptr(colsum),
                             _stream(stream)), "cwac_colsum")


# --------------------------------------------------------------------------- calibration
def cwac_stats_bytes(c_out: int) -> int:
    return int(lib().cwac_stats_bytes(c_out))


def cwac_stats_reset(stats: torch.Tensor, c_out: int, stream=None):
    _check(lib().cwac_stats_reset(_ptr(stats), c_out, _stream(stream)), "cwac_stats_reset")


def cwac_calibrate_stats_workspace(n_rows: int, c_out: int) -> int:
    return int(lib().cwac_calibrate_stats_workspace(n_rows, c_out))


def cwac_calibrate_stats(y_full: torch.Tensor, y_quant: torch.Tensor, stats: torch.Tensor,
                         workspace: torch.Tensor, stream=None, first: bool = False):
    """first=True calls cwac_calibrate_stats_first (the state is taken as empty: no reset needed)."""
    assert y_full.dtype == torch.float32 and y_quant.dtype == torch.float32
    assert y_full.shape == y_quant.shape
    n_rows, c_out = y_full.shape
    fn = lib().cwac_calibrate_stats_first if first else lib().cwac_calibrate_stats
    _check(fn(_ptr(y_full), _rowmajor(y_full), _ptr(y_quant), _rowmajor(y_quant), n_rows, c_out,
              _ptr(stats), _ptr(workspace), workspace.numel() * workspace.element_size(),
              _stream(stream)), "cwac_calibrate_stats_first" if first else "cwac_calibrate_stats")


def cwac_static_scratch_bytes() -> int:
    return int(lib().cwac_static_scratch_bytes())


def cwac_calibrate_stats_static(y_full: torch.Tensor, y_quant: torch.Tensor, stats: torch.Tensor,
                                stream=None):
    """cwac_calibrate_stats on the library's own fixed scratch buffer: no workspace, no allocation."""
    assert y_full.dtype == torch.float32 and y_quant.dtype == torch.float32
    assert y_full.shape == y_quant.shape
    n_rows, c_out = y_full.shape
    _check(lib().cwac_calibrate_stats_static(_ptr(y_full), _rowmajor(y_full), _ptr(y_quant),
                                             _rowmajor(y_quant), n_rows, c_out, _ptr(stats),
                                             _stream(stream)), "cwac_calibrate_stats_static")


def cwac_calibrate_stats_first(y_full, y_quant, stats, workspace, stream=None):
    cwac_calibrate_stats(y_full, y_quant, stats, workspace, stream, first=True)


def cwac_solve(stats: torch.Tensor, c_out: int, alpha: torch.Tensor, beta: torch.Tensor,
               moments: Optional[torch.Tensor] = None, n_degenerate: Optional[torch.Tensor] = None,
               var_eps: float = 1e-12, stream=None):
    assert alpha.dtype == torch.float32 and beta.dtype == torch.float32
    assert moments is None or (moments.dtype == torch.float64 and moments.numel() == 5 * c_out)
    _check(lib().cwac_solve(_ptr(stats), c_out, var_eps, _ptr(alpha), _ptr(beta), _ptr(moments),
                            _ptr(n_degenerate), _stream(stream)), "cwac_solve")


# --------------------------------------------------------------------------- fold
def cwac_fold(alpha, beta, s_w, bias, colsum, qp: cwac_qparams, mult, offset, fbias=None,
              n_saturated=None, stream=None):
    _check(lib().cwac_fold(_ptr(alpha), _ptr(beta), _ptr(s_w), _ptr(bias), _ptr(colsum),
                           s_w.numel(), C.byref(qp), _ptr(mult), _ptr(offset), _ptr(fbias),
                           _ptr(n_saturated), _stream(stream)), "cwac_fold")


# --------------------------------------------------------------------------- forward
_OUT_DTYPE = {CWAC_OUT_INT8: torch.int8, CWAC_OUT_FP32: torch.float32, CWAC_OUT_INT32: torch.int32}


def qlinear_cwac_forward(x_q: torch.Tensor, w_q: torch.Tensor, qp: Optional[cwac_qparams], mult,
                         offset, fbias, s_x_row, out_kind: int, out: torch.Tensor, stream=None,
                         tuning: Optional[cwac_tuning] = None):
    """tuning given: qlinear_cwac_forward_ex (the forward calls below likewise)."""
    assert x_q.dtype == torch.int8 and w_q.dtype == torch.int8
    assert out.dtype == _OUT_DTYPE[out_kind]
    m, k = x_q.shape
    n, k2 = w_q.shape
    assert k == k2 and out.shape == (m, n)
    args = (_ptr(x_q), _rowmajor(x_q), _ptr(w_q), _rowmajor(w_q), m, n, k,
            C.byref(qp) if qp is not None else None, _ptr(mult), _ptr(offset), _ptr(fbias),
            _ptr(s_x_row), out_kind, _ptr(out), _rowmajor(out))
    if tuning is None:
        _check(lib().qlinear_cwac_forward(*args, _stream(stream)), "qlinear_cwac_forward")
    else:
        _check(lib().qlinear_cwac_forward_ex(*args, _tun(tuning), _stream(stream)),
               "qlinear_cwac_forward_ex")


def qlinear_cwac_forward_table(x_q: torch.Tensor, w_q: torch.Tensor, qp: cwac_qparams, mult, offset,
                               table: torch.Tensor, out: torch.Tensor, stream=None, tuning=None):
    """int8 forward (integer-offset epilogue) with out = table[code + 128]."""
    assert x_q.dtype == torch.int8 and w_q.dtype == torch.int8 and out.dtype == torch.int8
    assert table.dtype == torch.int8 and table.numel() == 256
    m, k = x_q.shape
    n, k2 = w_q.shape
    assert k == k2 and out.shape == (m, n)
    args = (_ptr(x_q), _rowmajor(x_q), _ptr(w_q), _rowmajor(w_q), m, n, k, C.byref(qp), _ptr(mult),
            _ptr(offset), _ptr(table), _ptr(out), _rowmajor(out))
    if tuning is None:
        _check(lib().qlinear_cwac_forward_table(*args, _stream(stream)), "qlinear_cwac_forward_table")
    else:
        _check(lib().qlinear_cwac_forward_table_ex(*args, _tun(tuning), _stream(stream)),
               "qlinear_cwac_forward_table_ex")


def cwac_calibrate_fused_workspace(m: int, n: int) -> int:
    return int(lib().cwac_calibrate_fused_workspace(m, n))


def qlinear_cwac_calibrate_fused(x_q: torch.Tensor, w_q: torch.Tensor, mult, offset, fbias, s_x_row,
                                 y_full: torch.Tensor, stats: torch.Tensor,
                                 workspace: torch.Tensor, stream=None, tuning=None):
    assert x_q.dtype == torch.int8 and w_q.dtype == torch.int8 and y_full.dtype == torch.float32
    m, k = x_q.shape
    n, k2 = w_q.shape
    assert k == k2 and y_full.shape == (m, n)
    args = (_ptr(x_q), _rowmajor(x_q), _ptr(w_q), _rowmajor(w_q), m, n, k, _ptr(mult), _ptr(offset),
            _ptr(fbias), _ptr(s_x_row), _ptr(y_full), _rowmajor(y_full), _ptr(stats), _ptr(workspace),
            workspace.numel() * workspace.element_size())
    if tuning is None:
        _check(lib().qlinear_cwac_calibrate_fused(*args, _stream(stream)), "qlinear_cwac_calibrate_fused")
    else:
        _check(lib().qlinear_cwac_calibrate_fused_ex(*args, _tun(tuning), _stream(stream)),
               "qlinear_cwac_calibrate_fused_ex")


def cwac_epilogue_int32(acc: torch.Tensor, qp, mult, offset, fbias, s_x_row, out_kind: int,
                        out: torch.Tensor, stream=None):
    assert acc.dtype == torch.int32 and out.dtype == _OUT_DTYPE[out_kind]
    m, n = acc.shape
    _check(lib().cwac_epilogue_int32(_ptr(acc), _rowmajor(acc), m, n,
                                     C.byref(qp) if qp is not None else None, _ptr(mult),
                                     _ptr(offset), _ptr(fbias), _ptr(s_x_row), out_kind, _ptr(out),
                                     _rowmajor(out), _stream(stream)), "cwac_epilogue_int32")


def cwac_apply_unfolded(y: torch.Tensor, alpha, beta, out: torch.Tensor, stream=None):
    assert y.dtype == torch.float32 and out.dtype == torch.float32 and y.shape == out.shape
    _check(lib().cwac_apply_unfolded(_ptr(y), _rowmajor(y), y.shape[0], y.shape[1], _ptr(alpha),
                                     _ptr(beta), _ptr(out), _rowmajor(out), _stream(stream)),
           "cwac_apply_unfolded")


# --------------------------------------------------------------------------- integer-only form
def cwac_fold_fixed_point(alpha, beta, s_w, bias, colsum, qp: cwac_qparams, m0, shift, offset,
                          n_saturated=None, stream=None):
    assert m0.dtype == torch.int32 and shift.dtype == torch.int32 and offset.dtype == torch.int32
    _check(lib().cwac_fold_fixed_point(_ptr(alpha), _ptr(beta), _ptr(s_w), _ptr(bias),
                                       _ptr(colsum), s_w.numel(), C.byref(qp), _ptr(m0),
                                       _ptr(shift), _ptr(offset), _ptr(n_saturated),
                                       _stream(stream)), "cwac_fold_fixed_point")


def qlinear_cwac_forward_fixed_point(x_q: torch.Tensor, w_q: torch.Tensor, qp: cwac_qparams, m0,
                                     shift, offset, out: torch.Tensor, stream=None, tuning=None):
    assert x_q.dtype == torch.int8 and w_q.dtype == torch.int8 and out.dtype == torch.int8
    assert m0.dtype == torch.int32 and shift.dtype == torch.int32
    m, k = x_q.shape
    n, k2 = w_q.shape
    assert k == k2 and out.shape == (m, n)
    args = (_ptr(x_q), _rowmajor(x_q), _ptr(w_q), _rowmajor(w_q), m, n, k, C.byref(qp), _ptr(m0),
            _ptr(shift), _ptr(offset), _ptr(out), _rowmajor(out))
    if tuning is None:
        _check(lib().qlinear_cwac_forward_fixed_point(*args, _stream(stream)),
               "qlinear_cwac_forward_fixed_point")
    else:
        _check(lib().qlinear_cwac_forward_fixed_point_ex(*args, _tun(tuning), _stream(stream)),
               "qlinear_cwac_forward_fixed_point_ex")


def qconv2d_cwac_forward(x_q: torch.Tensor, w_q: torch.Tensor, stride: int, pad: int,
                         qp: cwac_qparams, mult, offset, fbias, out_kind: int, out: torch.Tensor,
                         stream=None, tuning=None):
    """x_q int8 [B, H, W, C_in] (channels last), w_q int8 [C_out, KH, KW, C_in];
    out [B*OH*OW, C_out] int8 / float32 / int32 per out_kind."""
    assert x_q.dtype == torch.int8 and w_q.dtype == torch.int8
    assert x_q.is_contiguous() and w_q.is_contiguous() and x_q.dim() == 4 and w_q.dim() == 4
    b, h, w, c_in = x_q.shape
    c_out, kh, kw, c2 = w_q.shape
    assert c2 == c_in and out.shape[1] == c_out
    args = (_ptr(x_q), _ptr(w_q), b, h, w, c_in, c_out, kh, kw, stride, pad, C.byref(qp), _ptr(mult),
            _ptr(offset), _ptr(fbias), out_kind, _ptr(out), _rowmajor(out))
    if tuning is None:
        _check(lib().qconv2d_cwac_forward(*args, _stream(stream)), "qconv2d_cwac_forward")
    else:
        _check(lib().qconv2d_cwac_forward_ex(*args, _tun(tuning), _stream(stream)),
               "qconv2d_cwac_forward_ex")


# --------------------------------------------------------------------------- weight-only INT4
def cwac_w4_quantize_groupwise(w: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor,
                               zeros: torch.Tensor, stream=None):
    """scales: float16 [n, k/128] (the library sees the bit patterns)."""
    assert w.dtype == torch.float32 and codes.dtype == torch.uint8 and zeros.dtype == torch.uint8
    assert scales.dtype == torch.float16 and codes.is_contiguous() and codes.shape == w.shape
    n, k = w.shape
    assert scales.shape == (n, k // CWAC_W4_GROUP) and zeros.shape == scales.shape
    assert scales.is_contiguous() and zeros.is_contiguous()
    _check(lib().cwac_w4_quantize_groupwise(_ptr(w), _rowmajor(w), n, k, _ptr(codes), _ptr(scales),
                                            _ptr(zeros), _stream(stream)),
           "cwac_w4_quantize_groupwise")


def cwac_w4_packed_w_bytes(n: int, k: int) -> int:
    return int(lib().cwac_w4_packed_w_bytes(n, k))


def cwac_w4_pack(codes: torch.Tensor, scales: torch.Tensor, zeros: torch.Tensor,
                 packed_w: torch.Tensor, packed_sz: torch.Tensor, stream=None):
    assert codes.dtype == torch.uint8 and codes.is_contiguous() and zeros.dtype == torch.uint8
    assert scales.dtype == torch.float16 and scales.is_contiguous() and zeros.is_contiguous()
    n, k = codes.shape
    assert packed_w.numel() * packed_w.element_size() >= cwac_w4_packed_w_bytes(n, k)
    assert packed_sz.dtype in (torch.int32, torch.uint32) and packed_sz.numel() >= n * (k // CWAC_W4_GROUP)
    _check(lib().cwac_w4_pack(_ptr(codes), _ptr(scales), _ptr(zeros), n, k, _ptr(packed_w),
                              _ptr(packed_sz), _stream(stream)), "cwac_w4_pack")


def cwac_fold_weight_only(alpha, beta, bias, mult: torch.Tensor, fbias: torch.Tensor, stream=None):
    assert mult.dtype == torch.float32 and fbias.dtype == torch.float32
    _check(lib().cwac_fold_weight_only(_ptr(alpha), _ptr(beta), _ptr(bias), mult.numel(), _ptr(mult),
                                       _ptr(fbias), _stream(stream)), "cwac_fold_weight_only")


def qlinear_w4a16_cwac_forward(x: torch.Tensor, packed_w: torch.Tensor, packed_sz: torch.Tensor,
                               n: int, mult, fbias, out: torch.Tensor, stream=None, tuning=None):
    """x float16 [m, k]; out float16 (CWAC_OUT_FP16) or float32 (CWAC_OUT_FP32) [m, n]."""
    assert x.dtype == torch.float16 and out.dtype in (torch.float16, torch.float32)
    m, k = x.shape
    assert out.shape == (m, n)
    kind = CWAC_OUT_FP16 if out.dtype == torch.float16 else CWAC_OUT_FP32
    args = (_ptr(x), _rowmajor(x), _ptr(packed_w), _ptr(packed_sz), m, n, k, _ptr(mult), _ptr(fbias),
            kind, _ptr(out), _rowmajor(out))
    if tuning is None:
        _check(lib().qlinear_w4a16_cwac_forward(*args, _stream(stream)), "qlinear_w4a16_cwac_forward")
    else:
        _check(lib().qlinear_w4a16_cwac_forward_ex(*args, _tun(tuning), _stream(stream)),
               "qlinear_w4a16_cwac_forward_ex")


# --------------------------------------------------------------------------- block glue
def vit_residual_ln_quant(h: torch.Tensor, r, s_r: float, z_r: int, h_out, gamma, beta, eps: float,
                          s_x: float, z_x: int, x_q, stream=None):
    """h float16 [m, c]; r / x_q int8 [m, c] or None; h_out float16 [m, c] or None."""
    assert h.dtype == torch.float16
    m, c = h.shape
    _check(lib().vit_residual_ln_quant(_ptr(h), _rowmajor(h), _ptr(r), _rowmajor(r) if r is not None else 0,
                                       s_r, z_r, _ptr(h_out), _rowmajor(h_out) if h_out is not None else 0,
                                       _ptr(gamma), _ptr(beta), eps, s_x, z_x, _ptr(x_q),
                                       _rowmajor(x_q) if x_q is not None else 0, m, c, _stream(stream)),
           "vit_residual_ln_quant")


def vit_gelu_table(s_in: float, z_in: int, s_out: float, z_out: int, table: torch.Tensor, stream=None):
    assert table.dtype == torch.int8 and table.numel() == 256
    _check(lib().vit_gelu_table(s_in, z_in, s_out, z_out, _ptr(table), _stream(stream)), "vit_gelu_table")


def vit_table_lookup(x: torch.Tensor, table: torch.Tensor, out: torch.Tensor, stream=None):
    assert x.dtype == torch.int8 and out.dtype == torch.int8 and x.shape == out.shape
    _check(lib().vit_table_lookup(_ptr(x), _rowmajor(x), _ptr(table), _ptr(out), _rowmajor(out),
                                  x.shape[0], x.shape[1], _stream(stream)), "vit_table_lookup")


def vit_attention_int8(r_qkv: torch.Tensor, s: float, z: int, batch: int, tokens: int, heads: int,
                       s_a: float, z_a: int, a_q: torch.Tensor, head_dim: int = 64, bias=None, stream=None):
    """bias: None or float16 [heads, tokens, ldb] with ldb % 4 == 0, ldb >= tokens rounded up to 32."""
    assert r_qkv.dtype == torch.int8 and a_q.dtype == torch.int8
    c = head_dim * heads
    assert r_qkv.shape == (batch * tokens, 3 * c) and a_q.shape == (batch * tokens, c)
    ldb = 0
    if bias is not None:
        assert bias.dtype == torch.float16 and bias.is_contiguous() and bias.shape[:2] == (heads, tokens)
        ldb = bias.shape[2]
    _check(lib().vit_attention_int8(_ptr(r_qkv), _rowmajor(r_qkv), s, z, batch, tokens, heads, head_dim,
                                    _ptr(bias), ldb, s_a, z_a, _ptr(a_q), _rowmajor(a_q), _stream(stream)),
           "vit_attention_int8")


def vit_block_workspace(batch: int, tokens: int, heads: int, hidden: int) -> int:
    return int(lib().vit_block_workspace(batch, tokens, heads, hidden))


def make_block_params(batch, tokens, heads, hidden, eps, ln1, ln2, layers, gelu_table,
                      head_dim: int = 64, attn_bias=None) -> vit_block_params:
    """ln1 / ln2: (gamma, beta) device tensors; layers: four dicts with w_q, mult, offset (device
    tensors) and s_x, z_x, s_r, z_r.  The tensors must outlive the returned struct's use."""
    bp = vit_block_params()
    bp.batch, bp.tokens, bp.heads, bp.hidden, bp.eps = batch, tokens, heads, hidden, eps
    bp.ln1_gamma, bp.ln1_beta = ln1[0].data_ptr(), ln1[1].data_ptr()
    bp.ln2_gamma, bp.ln2_beta = ln2[0].data_ptr(), ln2[1].data_ptr()
    for i, ly in enumerate(layers):
        bp.layer[i].w_q = ly["w_q"].data_ptr()
        bp.layer[i].mult = ly["mult"].data_ptr()
        bp.layer[i].offset = ly["offset"].data_ptr()
        bp.layer[i].s_x, bp.layer[i].z_x = ly["s_x"], ly["z_x"]
        bp.layer[i].s_r, bp.layer[i].z_r = ly["s_r"], ly["z_r"]
    bp.gelu_table = gelu_table.data_ptr()
    bp.head_dim = head_dim
    if attn_bias is not None:
        assert attn_bias.dtype == torch.float16 and attn_bias.is_contiguous()
        bp.attn_bias, bp.attn_bias_ld = attn_bias.data_ptr(), attn_bias.shape[2]
    return bp


def vit_block_w8a8_forward(bp: vit_block_params, h: torch.Tensor, h_out: torch.Tensor,
                           workspace: torch.Tensor, stream=None):
    assert h.dtype == torch.float16 and h_out.dtype == torch.float16 and h.is_contiguous() and h_out.is_contiguous()
    assert h.shape == h_out.shape == (bp.batch * bp.tokens, (bp.head_dim or 64) * bp.heads)
    _check(lib().vit_block_w8a8_forward(C.byref(bp), _ptr(h), _ptr(h_out), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)),
           "vit_block_w8a8_forward")


def vit_encoder_w8a8_forward(blocks, h: torch.Tensor, h_out: torch.Tensor, workspace: torch.Tensor,
                             stream=None):
    """blocks: a sequence of vit_block_params of one shape; h_out may be h."""
    assert h.dtype == torch.float16 and h_out.dtype == torch.float16 and h.is_contiguous() and h_out.is_contiguous()
    arr = (vit_block_params * len(blocks))(*blocks)
    assert h.shape == h_out.shape == (arr[0].batch * arr[0].tokens, (arr[0].head_dim or 64) * arr[0].heads)
    _check(lib().vit_encoder_w8a8_forward(arr, len(blocks), _ptr(h), _ptr(h_out), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
           "vit_encoder_w8a8_forward")


def cwac_forward_kernel_for(m: int, n: int, k: int, ldx: int, ldw: int, out_kind: int = CWAC_OUT_INT8,
                            tuning: Optional[cwac_tuning] = None) -> int:
    """CWAC_KERNEL_* the forward would run for these sizes (host arithmetic only)."""
    r = int(lib().cwac_forward_kernel_for(m, n, k, ldx, ldw, out_kind, _tun(tuning)))
    _check(min(r, 0), "cwac_forward_kernel_for")
    return r


# --------------------------------------------------------------------------- _ex entry points
def _ex(fn):
    """The _ex entry point of a forward call: the same arguments with a cwac_tuning (an all-zero
    struct, i.e. the library's own choice, when none is given)."""
    def call(*args, tuning: Optional[cwac_tuning] = None, **kw):
        return fn(*args, tuning=tuning if tuning is not None else make_tuning(), **kw)
    call.__name__ = fn.__name__ + "_ex"
    call.__doc__ = fn.__doc__
    return call


qlinear_cwac_forward_ex = _ex(qlinear_cwac_forward)
qlinear_cwac_forward_table_ex = _ex(qlinear_cwac_forward_table)
qconv2d_cwac_forward_ex = _ex(qconv2d_cwac_forward)
qlinear_cwac_calibrate_fused_ex = _ex(qlinear_cwac_calibrate_fused)
qlinear_cwac_forward_fixed_point_ex = _ex(qlinear_cwac_forward_fixed_point)
qlinear_w4a16_cwac_forward_ex = _ex(qlinear_w4a16_cwac_forward)


# --------------------------------------------------------------------------- diagnostic
def cwac_mfma_probe(operands: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor,
                    stream=None) -> float:
    """Enqueues the register-resident MFMA loop; returns the int8 operations it performs."""
    assert operands.numel() * operands.element_size() >= 16384 and sink.dtype == torch.int32
    _check(lib().cwac_mfma_probe(_ptr(operands), iters, workgroups, _ptr(sink), _stream(stream)),
           "cwac_mfma_probe")
    return 2.0 * 32768 * 16 * iters * 4 * workgroups


def cwac_hbm_read_probe(src: torch.Tensor, workgroups: int, sink: torch.Tensor, stream=None) -> float:
    """Enqueues a read-only stream over `src`; returns the bytes it reads."""
    assert src.is_contiguous() and sink.dtype == torch.int32
    nbytes = src.numel() * src.element_size() // 16 * 16
    _check(lib().cwac_hbm_read_probe(_ptr(src), nbytes, workgroups, _ptr(sink), _stream(stream)),
           "cwac_hbm_read_probe")
    return float(nbytes)


def cwac_mfma_probe_f16(operands: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor,
                        stream=None) -> float:
    """Enqueues the register-resident binary16 MFMA loop; returns the floating-point operations it performs."""
    assert operands.dtype == torch.float16 and operands.numel() >= 8192 and sink.dtype == torch.int32
    _check(lib().cwac_mfma_probe_f16(_ptr(operands), iters, workgroups, _ptr(sink), _stream(stream)),
           "cwac_mfma_probe_f16")
    return 2.0 * 16384 * 16 * iters * 4 * workgroups


def cwac_kloop_probe(operands: torch.Tensor, panels: torch.Tensor, mode: int, stages: int, workgroups: int,
                     sink: torch.Tensor, stream=None) -> float:
    """Enqueues the forward tile's K loop with the ingredients of `mode` (0 MFMAs, 1 + LDS fragment reads,
    2 + stage barrier, 3 + panel stream, 4 the stream issued by four wavefronts); returns the int8 operations it performs."""
    assert operands.numel() * operands.element_size() >= 16384 and sink.dtype == torch.int32
    assert panels.numel() * panels.element_size() >= 65536
    _check(lib().cwac_kloop_probe(_ptr(operands), _ptr(panels), mode, stages, workgroups, _ptr(sink),
                                  _stream(stream)), "cwac_kloop_probe")
    return 2.0 * 32768 * 256 * stages * workgroups
