"""Pins for the oracle's fold (Sec. 3.4, Eq. 10-11) and engine forward (Eq. 7,
Eq. 10): exact rational arithmetic, the algebraic identities between the
folded and the unfolded layer, and the plain-PTQ special case."""
from fractions import Fraction

import numpy as np
import pytest

from cases import build_case


def _fr(v):
    return Fraction(float(v))


def _rne(fr: Fraction) -> int:
    return round(fr)            # Python rounds Fractions half-to-even


@pytest.fixture(scope="module")
def case1(orc):
    return build_case(orc, 1, m=48, cal_rows=256, n=64, k=96)


@pytest.fixture(scope="module")
def case5(orc):
    return build_case(orc, 5, m=40, cal_rows=192, n=48, k=256)


def test_fold_against_exact_rationals(orc, case1):
    c = case1
    mult, offset, nsat = orc.fold_int_offset(c.alpha, c.beta, c.sw, c.bias, c.colsum,
                                             c.sx, c.zx, c.sr)
    assert nsat == 0
    for ch in range(c.n):
        a, b = _fr(c.alpha[ch]), _fr(c.beta[ch])
        unit = _fr(c.sx) * _fr(c.sw[ch])
        m_exact = a * unit / _fr(c.sr)                       # Eq. 11
        ulp = _fr(np.spacing(np.float32(abs(mult[ch]))))
        assert abs(_fr(mult[ch]) - m_exact) <= ulp * Fraction(500001, 1000000)
        beta_q = _rne(b / (a * unit))                        # Eq. 10 integer offset
        bias_q = _rne(_fr(c.bias[ch]) / unit)                # engine's integer bias
        want = beta_q + bias_q - c.zx * int(c.colsum[ch])    # -Z_x W_q term of Eq. 7
        # fp64 evaluation may differ from the exact rational only at an exact tie
        assert abs(int(offset[ch]) - want) <= 0, (ch, int(offset[ch]), want)


def test_identity_fold_is_plain_ptq(orc, case1):
    """alpha = 1, beta = 0 turns Eq. 10-11 into Eq. 7-8: same parameters, same codes."""
    c = case1
    ones, zeros = np.ones(c.n, np.float32), np.zeros(c.n, np.float32)
    m0, o0, _ = orc.fold_int_offset(None, None, c.sw, c.bias, c.colsum, c.sx, c.zx, c.sr)
    m1, o1, _ = orc.fold_int_offset(ones, zeros, c.sw, c.bias, c.colsum, c.sx, c.zx, c.sr)
    np.testing.assert_array_equal(m0, m1)
    np.testing.assert_array_equal(o0, o1)
    for ch in range(c.n):                                    # Eq. 8: M = S_x S_W / S_r
        m_exact = _fr(c.sx) * _fr(c.sw[ch]) / _fr(c.sr)
        assert abs(_fr(m0[ch]) - m_exact) <= _fr(np.spacing(m0[ch])) * Fraction(500001, 1000000)
    r0 = orc.folded_forward(c.acc, o0, m0, c.zr)
    r1 = orc.folded_forward(c.acc, o1, m1, c.zr)
    np.testing.assert_array_equal(r0, r1)


def test_plain_ptq_forward_against_eq6(orc, case1):
    """Without bias and compensation the engine output is Eq. 6 solved for r_q:
    r_q = Z_r + round(S_W S_x sum_k W_q (x_q - Z_x) / S_r), clipped."""
    c = case1
    m0, o0, _ = orc.fold_int_offset(None, None, c.sw, None, c.colsum, c.sx, c.zx, c.sr)
    r = orc.folded_forward(c.acc, o0, m0, c.zr).astype(np.int64)
    t0 = (c.xq.astype(np.int64) - c.zx) @ c.wq.astype(np.int64).T
    v = t0 * (np.float64(c.sx) * c.sw.astype(np.float64) / np.float64(c.sr))[None, :] + c.zr
    inside = (v > -128) & (v < 127)
    assert inside.mean() > 0.5
    assert np.max(np.abs(r - v)[inside]) <= 0.5 + 1e-4
    assert np.all(r[v >= 127.5] == 127) and np.all(r[v <= -128.5] == -128)
    # a few elements in exact rationals, including the float conversion of the multiplier
    for (i, ch) in [(0, 0), (3, 7), (47, 63), (20, 31)]:
        u = int(t0[i, ch]) * _fr(m0[ch])
        want = min(127, max(-128, _rne(u) + c.zr))
        assert abs(int(r[i, ch]) - want) <= (1 if abs(u - _rne(u)) > Fraction(49, 100) else 0)


def test_ties_and_clamp(orc):
    acc = np.array([[1, 3, 5, -1, -3, 1000, -1000, 0]], dtype=np.int32)
    mult = np.full(8, 0.5, np.float32)
    off = np.zeros(8, np.int32)
    r = orc.folded_forward(acc, off, mult, 0)
    np.testing.assert_array_equal(r[0], [0, 2, 2, 0, -2, 127, -128, 0])   # half-to-even, clamp
    r = orc.folded_forward(acc, off, mult, 10)
    np.testing.assert_array_equal(r[0], [10, 12, 12, 10, 8, 127, -128, 10])
    r = orc.folded_forward(acc, off, mult, 0, qmin=-8, qmax=7)            # 4-bit codes in int8
    np.testing.assert_array_equal(r[0], [0, 2, 2, 0, -2, 7, -8, 0])
    big = np.array([[2**30 + 2**6 + 1]], dtype=np.int32)                   # int32 -> fp32 is RNE
    _, u = orc.folded_forward(big, np.zeros(1, np.int32), np.ones(1, np.float32), 0, want_f32=True)
    assert u[0, 0] == np.float32(2**30 + 2**7) or u[0, 0] == np.float32(2**30)
    assert u[0, 0] == np.float32(np.int32(2**30 + 2**6 + 1))


def test_folded_matches_unfolded_within_rounding(orc, case1):
    """Folding alpha is lossless, folding beta costs one rounding (two with the
    engine's integer bias): codes differ from the unfolded layer by at most
    floor(|M'| + 1), and rarely."""
    c = case1
    yq = orc.dequant_output(c.acc, c.colsum, c.zx, c.deq, c.bias)
    unf = orc.requant_output(orc.cwac_apply(yq, c.alpha, c.beta), c.sr, c.zr).astype(np.int64)
    fold = c.out.astype(np.int64)
    bound = np.floor(np.abs(c.mult.astype(np.float64)) + 1.0)[None, :]
    assert np.all(np.abs(fold - unf) <= bound)
    assert np.mean(fold != unf) < 0.25
    # against the real-valued unfolded code: |u_fold - u_unf| <= |M'| (two half-unit roundings)
    u_real = orc.unfolded_real(c.acc, c.colsum, c.zx, c.sw, c.sx, c.bias, c.alpha, c.beta, c.sr)
    _, u_fold = orc.folded_forward(c.acc, c.offset, c.mult, c.zr, want_f32=True)
    assert np.all(np.abs(u_fold - u_real) <= np.abs(c.mult)[None, :] * 1.0001 + 1e-4)


def test_fp_bias_matches_unfolded(orc, case1, case5):
    """Un-rounded beta: the folded layer differs from the unfolded one only by
    fp32 rounding, i.e. by at most one code and only next to a tie."""
    for c in (case5, build_case(orc, 1, m=48, cal_rows=256, n=64, k=96, fp_bias=True)):
        yq = orc.dequant_output(c.acc, c.colsum, c.zx, c.deq, c.bias, c.sx_row)
        unf = orc.requant_output(orc.cwac_apply(yq, c.alpha, c.beta), c.sr, c.zr).astype(np.int64)
        fold = c.out.astype(np.int64)
        assert np.max(np.abs(fold - unf)) <= 1
        assert np.mean(fold != unf) < 0.01
        u_real = orc.unfolded_real(c.acc, c.colsum, c.zx, c.sw, c.sx, c.bias, c.alpha, c.beta,
                                   c.sr, c.sx_row)
        _, u_fold = orc.folded_forward(c.acc, c.offset, c.mult, c.zr, c.fbias, c.sx_row,
                                       want_f32=True)
        assert np.max(np.abs(u_fold - u_real) / (1 + np.abs(u_real))) < 1e-5


def test_calibration_output_is_the_fp_bias_epilogue(orc, case1, case5):
    """Y_quant (dequantized module output) is the folded forward with alpha = 1,
    beta = 0, S_r = 1 and the un-rounded value kept."""
    for c in (case1, case5):
        mult, fbias, off = orc.fold_fp_bias(None, None, c.sw, c.bias, c.colsum, c.per_token,
                                            c.sx, c.zx, 1.0)
        np.testing.assert_array_equal(mult, c.deq)
        if c.bias is not None:
            np.testing.assert_array_equal(fbias, c.bias)
        _, u = orc.folded_forward(c.acc_cal, off, mult, 0, fbias if c.bias is not None else None,
                                  c.sx_row_cal, want_f32=True)
        np.testing.assert_array_equal(u, c.y_quant)
        # and it approximates the full-precision output (quantization noise only)
        err = np.abs(c.y_quant - c.y_full).mean() / np.abs(c.y_full).mean()
        assert err < 0.2


def test_compensation_reduces_error(orc, case1):
    """The fitted affine cannot be worse than the identity on its own calibration set."""
    c = case1
    yc = orc.cwac_apply(c.y_quant, c.alpha, c.beta).astype(np.float64)
    e0 = ((c.y_quant.astype(np.float64) - c.y_full) ** 2).sum(0)
    e1 = ((yc - c.y_full) ** 2).sum(0)
    assert np.all(e1 <= e0 * (1 + 1e-6) + 1e-9)


def test_offset_saturation(orc, case1):
    c = case1
    alpha = c.alpha.copy()
    alpha[3] = 1e-30                                       # beta / (alpha S_x S_W) overflows int32
    alpha[4] = -1e-30
    mult, offset, nsat = orc.fold_int_offset(alpha, c.beta, c.sw, c.bias, c.colsum,
                                             c.sx, c.zx, c.sr)
    assert nsat == 2
    sgn = np.sign(c.beta[3])
    assert offset[3] + c.zx * c.colsum[3] == int(sgn) * 2**30
    assert offset[4] + c.zx * c.colsum[4] == -int(np.sign(c.beta[4])) * 2**30
    r = orc.folded_forward(c.acc, offset, mult, c.zr)      # no int32 wrap, finite codes
    assert r.dtype == np.int8
