"""GPU parity at low bit widths (W4A4, W6A6; codes in int8 containers): the b-bit quantizers and
the whole pipeline - calibration forward, statistics, fit, fold, folded forward with a b-bit
output range - against the oracle, through the C ABI."""

import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth
from tuning import tuning_of

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-5


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


@pytest.mark.parametrize("bits", [2, 4, 6, 8])
def test_low_bit_quantizers(orc, bits):
    half = 1 << (bits - 1)
    for rows, k in ((37, 77), (64, 256)):              # element-wise and vector paths
        x = (2.0 * synth.normal(7300 + bits, 0, rows * k).numpy()).reshape(rows, k).astype(np.float32)
        x[3] = 0.0
        mn, mx = orc.range_f32(x)
        s, z_u = orc.qparams_asym(mn, mx, bits)
        s2, z2 = P.cwac_qparams_from_range(float(mn), float(mx), bits)
        assert (np.float32(s2), z2) == (s, z_u)
        q = torch.empty(rows, k, dtype=torch.int8, device=DEV)
        P.cwac_quantize_act_bits(dev(x), float(s), z_u - half, bits, q)
        np.testing.assert_array_equal(host(q), orc.quantize_act_bits(x, s, z_u - half, bits))
        sc = torch.empty(rows, dtype=torch.float32, device=DEV)
        P.cwac_quantize_rows_sym_bits(dev(x), bits, sc, q)
        q0, s0 = orc.quantize_rows_sym_bits(x, bits)
        np.testing.assert_array_equal(host(q), q0)
        np.testing.assert_array_equal(host(sc), s0)
    with pytest.raises(P.CwacError):
        P.cwac_quantize_act_bits(dev(x), 1.0, half, bits, q)          # zero-point outside the range
    with pytest.raises(P.CwacError):
        P.cwac_quantize_rows_sym_bits(dev(x), 9, sc, q)


@pytest.mark.parametrize("bits,fast", [(4, False), (6, False), (4, True)])
def test_low_bit_pipeline(orc, bits, fast):
    """ViT-shaped layer (workload 1's recipe) at W{bits}A{bits}: every stage on the device against
    the oracle.  fast: a size the large-problem kernel takes."""
    wl = synth.WORKLOADS[1]
    half, qmin, qmax = 1 << (bits - 1), -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    m, cal = (512, 768) if fast else (197, 1024)
    _pipeline(orc, wl, bits, half, qmin, qmax, m, cal, tuning_of("fast") if fast else None)


def _pipeline(orc, wl, bits, half, qmin, qmax, m, cal, tun=None):
    w_t, b_t = synth.weights(wl, 0)
    w, bias = w_t.numpy(), b_t.numpy()
    n, k = w.shape
    x = synth.activations(wl, 0, m).numpy()
    xcal = synth.activations(wl, 0, cal, calibration=True).numpy()
    yf = (xcal @ w.T + bias).astype(np.float32)
    # ---- oracle
    wq0, sw0 = orc.quantize_rows_sym_bits(w, bits)
    cs0 = orc.colsum_i8(wq0)
    mn, mx = orc.range_f32(xcal)
    s0, z_u = orc.qparams_asym(mn, mx, bits)
    zx = z_u - half
    xq0, xqc0 = orc.quantize_act_bits(x, s0, zx, bits), orc.quantize_act_bits(xcal, s0, zx, bits)
    yq0 = orc.dequant_output(orc.gemm_i8(xqc0, wq0), cs0, zx, orc.deq_scale(sw0, s0), bias, None)
    mom0 = orc.channel_moments(yf, yq0)
    a0, b0, _ = orc.solve(mom0)
    yc = orc.cwac_apply(yq0, a0, b0)
    sr0, zr_u = orc.qparams_asym(*orc.range_f32(yc), bits)
    zr = zr_u - half
    # ---- device
    wq = torch.empty(n, k, dtype=torch.int8, device=DEV)
    sw = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_quantize_rows_sym_bits(dev(w), bits, sw, wq)
    colsum = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_colsum(wq, colsum)
    xq = torch.empty(m, k, dtype=torch.int8, device=DEV)
    xqc = torch.empty(cal, k, dtype=torch.int8, device=DEV)
    P.cwac_quantize_act_bits(dev(x), float(s0), zx, bits, xq)
    P.cwac_quantize_act_bits(dev(xcal), float(s0), zx, bits, xqc)
    np.testing.assert_array_equal(host(wq), wq0)
    np.testing.assert_array_equal(host(xq), xq0)
    np.testing.assert_array_equal(host(colsum), cs0)
    f32 = dict(dtype=torch.float32, device=DEV)
    dm, dfb = torch.empty(n, **f32), torch.empty(n, **f32)
    do = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_fold(None, None, sw, dev(bias), colsum,
                P.make_qparams(P.CWAC_EPI_FP_BIAS, False, float(s0), zx, 1.0, 0), dm, do, dfb)
    yq = torch.empty(cal, n, **f32)
    P.qlinear_cwac_forward(xqc, wq, None, dm, do, dfb, None, P.CWAC_OUT_FP32, yq, tuning=tun)
    np.testing.assert_array_equal(host(yq), yq0)
    st = torch.empty(P.cwac_stats_bytes(n) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, n)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(cal, n), dtype=torch.uint8, device=DEV)
    P.cwac_calibrate_stats(dev(yf), yq, st, ws)
    alpha, beta = torch.empty(n, **f32), torch.empty(n, **f32)
    P.cwac_solve(st, n, alpha, beta)
    a, b = host(alpha), host(beta)
    sf = np.sqrt(mom0[4])
    assert np.max(np.abs(a - a0) / np.maximum(np.abs(a0), 1.0)) <= RTOL
    assert np.max(np.abs(b - b0) / np.maximum(np.abs(b0), sf)) <= RTOL
    # fold and folded forward with the device's own (alpha, beta): compare with the oracle's fold
    # of the SAME fp32 values, then its epilogue, with the b-bit output range
    qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, float(s0), zx, float(sr0), zr, qmin, qmax)
    mult, off = torch.empty(n, **f32), torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_fold(alpha, beta, sw, dev(bias), colsum, qp, mult, off)
    m1, o1, _ = orc.fold_int_offset(a, b, sw0, bias, cs0, s0, zx, sr0)
    np.testing.assert_array_equal(host(mult), m1)
    np.testing.assert_array_equal(host(off), o1)
    out = torch.empty(m, n, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward(xq, wq, qp, mult, off, None, None, P.CWAC_OUT_INT8, out, tuning=tun)
    acc = orc.gemm_i8(xq0, wq0)
    want = orc.folded_forward(acc, o1, m1, zr, None, None, qmin, qmax)
    got = host(out)
    np.testing.assert_array_equal(got, want)
    assert got.min() >= qmin and got.max() <= qmax and len(np.unique(got)) > (1 << bits) // 2
    # the integer-only epilogue at the same bit width
    m0 = torch.empty(n, dtype=torch.int32, device=DEV)
    sh = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_fold_fixed_point(alpha, beta, sw, dev(bias), colsum, qp, m0, sh, off)
    P.qlinear_cwac_forward_fixed_point(xq, wq, qp, m0, sh, off, out, tuning=tun)
    q0, s1, o2, _ = orc.fold_fixed_point(a, b, sw0, bias, cs0, s0, zx, sr0)
    np.testing.assert_array_equal(host(out), orc.fixed_point_forward(acc, o2, q0, s1, zr, qmin, qmax))
