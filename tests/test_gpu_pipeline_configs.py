"""The whole calibrated pipeline of every workload, stage by stage against the oracle, at the
layers' true N and K on each workload's own activation statistics:

    quantizers -> calibration forward (fp32 Y_quant) -> statistics in two uneven batches
    (reset-free first batch) -> closed-form fit -> fold -> compensated int8 forward,

plus the same calibration side as one call (statistics in the calibration GEMM's epilogue).
Token and calibration row counts are cut so that the oracle finishes in seconds (the full-size
launches are checked on sampled rows in test_gpu_full_size.py); both are ragged: several tiles
and a tail.  Integers bit for bit; moments and (alpha, beta) within 1e-5 relative."""
import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from cases import build_case

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-5

# (workload, layer index, inference rows, calibration rows)
CASES = [(2, 0, 1333, 4099),
         (3, 0, 1333, 4099), (3, 1, 1333, 4099), (3, 2, 1333, 4099), (3, 3, 1333, 4099),
         (4, 0, 1333, 4099), (4, 1, 1333, 4099), (4, 2, 1333, 4099),
         (5, 0, 515, 2055), (5, 4, 515, 2055)]


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def _check_moments(mom, ref):
    sf, sq = np.sqrt(ref[4]), np.sqrt(ref[2])
    floors = [sf, sq, sq * sq, sq * sf, sf * sf]
    for i in range(5):
        err = np.abs(mom[i] - ref[i]) / (np.maximum(np.abs(ref[i]), floors[i]) + 1e-300)
        assert err.max() <= RTOL, (i, err.max())


def _check_fit(alpha, beta, c):
    sf = np.sqrt(c.moments[4])
    assert np.max(np.abs(alpha - c.alpha) / np.maximum(np.abs(c.alpha), 1.0)) <= RTOL
    assert np.max(np.abs(beta - c.beta) / np.maximum(np.abs(c.beta), sf)) <= RTOL


def _solve(st, n):
    alpha = torch.empty(n, dtype=torch.float32, device=DEV)
    beta = torch.empty(n, dtype=torch.float32, device=DEV)
    mom = torch.empty(5, n, dtype=torch.float64, device=DEV)
    ndeg = torch.zeros(1, dtype=torch.int32, device=DEV)
    P.cwac_solve(st, n, alpha, beta, mom, ndeg)
    return alpha, beta, host(mom), int(host(ndeg)[0])


@pytest.mark.parametrize("cfg,layer,m,cal_rows", CASES)
def test_calibrated_pipeline(orc, cfg, layer, m, cal_rows):
    c = build_case(orc, cfg, layer, m=m, cal_rows=cal_rows)
    n, k, per_token = c.n, c.k, c.per_token
    print(f"config {cfg} layer {layer}: {m} rows, {cal_rows} calibration rows, {n} x {k}, "
          f"per_token={per_token}", flush=True)
    f32 = dict(dtype=torch.float32, device=DEV)
    i32 = dict(dtype=torch.int32, device=DEV)

    # ---- quantizers (Eq. 1-2)
    wq = torch.empty(n, k, dtype=torch.int8, device=DEV)
    sw = torch.empty(n, **f32)
    P.cwac_quantize_rows_sym(dev(c.w), sw, wq)
    colsum = torch.empty(n, **i32)
    P.cwac_colsum(wq, colsum)
    np.testing.assert_array_equal(host(wq), c.wq)
    np.testing.assert_array_equal(host(sw), c.sw)
    np.testing.assert_array_equal(host(colsum), c.colsum)
    xq = torch.empty(m, k, dtype=torch.int8, device=DEV)
    xq_cal = torch.empty(cal_rows, k, dtype=torch.int8, device=DEV)
    if per_token:
        sx_row, sx_row_cal = torch.empty(m, **f32), torch.empty(cal_rows, **f32)
        P.cwac_quantize_rows_sym(dev(c.x), sx_row, xq)
        P.cwac_quantize_rows_sym(dev(c.xcal), sx_row_cal, xq_cal)
        np.testing.assert_array_equal(host(sx_row), c.sx_row)
        np.testing.assert_array_equal(host(sx_row_cal), c.sx_row_cal)
        sx, zx = 1.0, 0
    else:
        xcal = dev(c.xcal)
        mm = torch.empty(2, **f32)
        ws = torch.empty(P.cwac_range_workspace(xcal.numel()), dtype=torch.uint8, device=DEV)
        P.cwac_range_f32(xcal, mm, ws)
        mn, mx = host(mm)
        sx, z_u = P.cwac_qparams_from_range(float(mn), float(mx), 8)
        zx = z_u - 128
        assert (np.float32(sx), zx) == (c.sx, c.zx)
        P.cwac_quantize_act(dev(c.x), sx, zx, xq)
        P.cwac_quantize_act(xcal, sx, zx, xq_cal)
        sx_row = sx_row_cal = None
    np.testing.assert_array_equal(host(xq), c.xq)
    np.testing.assert_array_equal(host(xq_cal), c.xq_cal)
    bias = dev(c.bias)

    # ---- calibration forward: Y_quant of Sec. 3.3, bit for bit
    dm, dfb = torch.empty(n, **f32), torch.empty(n, **f32)
    do = torch.empty(n, **i32)
    P.cwac_fold(None, None, sw, bias, colsum, P.make_qparams(P.CWAC_EPI_FP_BIAS, per_token, sx, zx, 1.0, 0),
                dm, do, dfb)
    np.testing.assert_array_equal(host(dm), c.deq)
    dfb_arg = dfb if bias is not None else None
    yq = torch.empty(cal_rows, n, **f32)
    P.qlinear_cwac_forward(xq_cal, wq, None, dm, do, dfb_arg, sx_row_cal, P.CWAC_OUT_FP32, yq)
    np.testing.assert_array_equal(host(yq), c.y_quant)

    # ---- statistics (Eq. 4-5 sums) in two uneven batches; the first needs no reset: the state starts
    # as garbage on purpose
    yf = dev(c.y_full)
    cut = cal_rows // 2 - 3
    st = torch.full((P.cwac_stats_bytes(n) // 8 + 2,), float("nan"), dtype=torch.float64, device=DEV)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(cal_rows, n), dtype=torch.uint8, device=DEV)
    P.cwac_calibrate_stats_first(yf[:cut], yq[:cut], st, ws)
    P.cwac_calibrate_stats(yf[cut:], yq[cut:], st, ws)
    assert int(host(st.view(torch.int64)[:1])[0]) == cal_rows
    alpha, beta, mom, ndeg = _solve(st, n)
    _check_moments(mom, c.moments)
    a, b = host(alpha), host(beta)
    _check_fit(a, b, c)
    assert ndeg == c.n_degenerate
    # the reset + accumulate form of the same two batches leaves the same state, bit for bit
    st_r = torch.empty_like(st)
    P.cwac_stats_reset(st_r, n)
    P.cwac_calibrate_stats(yf[:cut], yq[:cut], st_r, ws)
    P.cwac_calibrate_stats(yf[cut:], yq[cut:], st_r, ws)
    words = P.cwac_stats_bytes(n) // 8
    assert torch.equal(st[:words].view(torch.int64), st_r[:words].view(torch.int64))

    # ---- the calibration side as one call per batch (statistics in the GEMM's epilogue)
    st_f = torch.empty_like(st)
    P.cwac_stats_reset(st_f, n)
    wsf = torch.empty(P.cwac_calibrate_fused_workspace(cal_rows, n), dtype=torch.uint8, device=DEV)
    for lo, hi in ((0, cut), (cut, cal_rows)):
        P.qlinear_cwac_calibrate_fused(xq_cal[lo:hi], wq, dm, do, dfb_arg,
                                       None if sx_row_cal is None else sx_row_cal[lo:hi], yf[lo:hi], st_f, wsf)
    alpha_f, beta_f, mom_f, _ = _solve(st_f, n)
    _check_moments(mom_f, c.moments)
    _check_fit(host(alpha_f), host(beta_f), c)

    # ---- fold (Eq. 10-11) of the DEVICE's (alpha, beta): the oracle folds the same fp32 values
    mult, fb = torch.empty(n, **f32), torch.empty(n, **f32)
    off = torch.empty(n, **i32)
    nsat = torch.zeros(1, **i32)
    if c.fp_bias:
        qp = P.make_qparams(P.CWAC_EPI_FP_BIAS, per_token, sx, zx, c.sr, c.zr)
        P.cwac_fold(alpha, beta, sw, bias, colsum, qp, mult, off, fb, nsat)
        m0, b0, o0 = orc.fold_fp_bias(a, b, c.sw, c.bias, c.colsum, per_token, c.sx, c.zx, c.sr)
        np.testing.assert_array_equal(host(fb), b0)
    else:
        qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, sx, zx, c.sr, c.zr)
        P.cwac_fold(alpha, beta, sw, bias, colsum, qp, mult, off, None, nsat)
        m0, o0, ns0 = orc.fold_int_offset(a, b, c.sw, c.bias, c.colsum, c.sx, c.zx, c.sr)
        b0 = None
        assert int(host(nsat)[0]) == ns0
    np.testing.assert_array_equal(host(mult), m0)
    np.testing.assert_array_equal(host(off), o0)

    # ---- compensated int8 forward (Eq. 10), bit for bit
    out = torch.empty(m, n, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward(xq, wq, qp, mult, off, fb if c.fp_bias else None, sx_row, P.CWAC_OUT_INT8, out)
    got = host(out)
    np.testing.assert_array_equal(got, orc.folded_forward(c.acc, o0, m0, c.zr, b0, c.sx_row))
    # against the oracle's own end-to-end codes: (alpha, beta) within 1e-5 move a code only next to
    # a rounding boundary
    diff = got.astype(np.int32) - c.out.astype(np.int32)
    assert np.max(np.abs(diff)) <= 1 and np.mean(diff != 0) < 1e-3
    assert len(np.unique(got)) > 32, "the output codes should spread over the range"
