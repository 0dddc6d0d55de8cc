"""Pins of the oracle's b-bit quantizers (codes in int8 containers; the W4A4 / W6A6 settings of
the paper's tables): exact rational arithmetic, agreement with the unsigned Eq. 1 form, range
ends; and the method's guarantee at low bit widths (compensation never increases the
calibration error)."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2505_20932_amd import synth


@pytest.mark.parametrize("bits", [2, 4, 6, 8])
def test_act_bits_is_eq1_shifted_by_half_range(orc, bits):
    x = (3.0 * synth.normal(7100 + bits, 0, 4000).numpy()).astype(np.float32)
    x[:4] = [x.min() - 5.0, x.max() + 5.0, 0.0, -0.0]
    mn, mx = orc.range_f32(x[4:])
    s, z_u = orc.qparams_asym(mn, mx, bits)
    half = 1 << (bits - 1)
    q = orc.quantize_act_bits(x, s, z_u - half, bits)
    # the unsigned form (pinned on its own against Eq. 1) shifted by 2^(bits-1)
    np.testing.assert_array_equal(q.astype(np.int32) + half, orc.quantize_asym(x, s, z_u, bits))
    assert q.min() == -half and q.max() == half - 1          # both clip ends are reached
    # every code is the nearest integer to the exact quotient (fp32 division is correctly rounded,
    # so check against the rational value of fl(x / s))
    for i in range(0, 4000, 37):
        quo = Fraction(float(np.float32(x[i]) / np.float32(s)))
        r = round(quo)                                            # ties to even, like rint
        want = min(max(r + z_u, 0), 2 ** bits - 1) - half
        assert int(q[i]) == want
    if bits == 8:
        np.testing.assert_array_equal(q, orc.quantize_act_i8(x, s, z_u - half))


@pytest.mark.parametrize("bits", [2, 4, 6, 8])
def test_rows_sym_bits(orc, bits):
    rows, k = 9, 333
    x = synth.normal(7200 + bits, 0, rows * k).numpy().reshape(rows, k).astype(np.float32)
    x[4] = 0.0
    q, s = orc.quantize_rows_sym_bits(x, bits)
    qmax = 2 ** (bits - 1) - 1
    for r in range(rows):
        amax = np.abs(x[r]).max()
        if amax == 0:
            assert np.all(q[r] == 0) and s[r] > 0
            continue
        assert s[r] == np.float32(amax) / np.float32(qmax)
        assert np.abs(q[r]).max() == qmax and q[r].min() >= -qmax      # -2^(b-1) never used
        for j in range(0, k, 11):
            quo = Fraction(float(np.float32(x[r, j]) / s[r]))
            assert int(q[r, j]) == min(max(round(quo), -qmax), qmax)
    q2, s2 = orc.quantize_rows_sym_bits(-x, bits)                       # odd symmetry
    np.testing.assert_array_equal(q2, -q)
    np.testing.assert_array_equal(s2, s)
    if bits == 8:
        q8, s8 = orc.quantize_rows_sym(x)
        np.testing.assert_array_equal(q, q8)
        np.testing.assert_array_equal(s, s8)


@pytest.mark.parametrize("bits", [4, 6])
def test_compensation_at_low_bits(orc, bits):
    """Sec. 3.3: the least-squares (alpha, beta) cannot increase the calibration error of any
    channel; at low bit widths the quantization error it works on is large."""
    wl = synth.WORKLOADS[1]
    w_t, b_t = synth.weights(wl, 0)
    w, bias = w_t.numpy(), b_t.numpy()
    x = synth.activations(wl, 0, 2048, calibration=True).numpy()
    yf = (x @ w.T + bias).astype(np.float32)
    half = 1 << (bits - 1)
    wq, sw = orc.quantize_rows_sym_bits(w, bits)
    mn, mx = orc.range_f32(x)
    s, z_u = orc.qparams_asym(mn, mx, bits)
    zx = z_u - half
    xq = orc.quantize_act_bits(x, s, zx, bits)
    acc = orc.gemm_i8(xq, wq)
    assert np.abs(acc).max() <= x.shape[1] * half * (half - 1)
    yq = orc.dequant_output(acc, orc.colsum_i8(wq), zx, orc.deq_scale(sw, s), bias, None)
    alpha, beta, _ = orc.solve(orc.channel_moments(yf, yq))
    yc = orc.cwac_apply(yq, alpha, beta)
    e0 = np.mean((yq.astype(np.float64) - yf) ** 2, axis=0)
    e1 = np.mean((yc.astype(np.float64) - yf) ** 2, axis=0)
    assert np.all(e1 <= e0 * (1 + 1e-5))
    assert e1.sum() < 0.99 * e0.sum()
    e8 = None
    if bits == 4:   # the error being compensated is far larger than at 8 bits
        wq8, sw8 = orc.quantize_rows_sym(w)
        s8, z8 = orc.qparams_asym(mn, mx, 8)
        xq8 = orc.quantize_act_i8(x, s8, z8 - 128)
        yq8 = orc.dequant_output(orc.gemm_i8(xq8, wq8), orc.colsum_i8(wq8), z8 - 128,
                                 orc.deq_scale(sw8, s8), bias, None)
        e8 = np.mean((yq8.astype(np.float64) - yf) ** 2)
        assert e0.mean() > 20 * e8
