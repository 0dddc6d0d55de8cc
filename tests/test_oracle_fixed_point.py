"""Pins of the oracle's integer-only engine form (multiplier M' of Eq. 11 as M0 * 2^-shift,
epilogue of Eq. 10 in 64-bit integer arithmetic): exact rational arithmetic with Python integers
and fractions, range edge cases, and the relation to the fp32 epilogue."""
from fractions import Fraction

import numpy as np

from paper_2505_20932_amd import synth


def _real_multiplier(a, sx, sw, sr):
    """alpha * S_x * S_W / S_r of fp32 inputs as an exact rational."""
    return Fraction(float(a)) * Fraction(float(sx)) * Fraction(float(sw)) / Fraction(float(sr))


def test_multiplier_has_31_significant_bits(orc):
    n = 400
    g = synth.normal(9001, 0, 3 * n).numpy().astype(np.float64)
    alpha = (np.sign(g[:n]) * np.exp(2.0 * g[:n])).astype(np.float32)          # both signs, wide range
    sw = np.exp(-4.0 + g[n:2 * n]).astype(np.float32)
    sx, sr = np.float32(0.0123), np.float32(0.37)
    m0, sh, off, nsat = orc.fold_fixed_point(alpha, None, sw, None, np.zeros(n, np.int32), sx, 0, sr)
    assert nsat == 0 and np.all(off == 0)
    for c in range(n):
        real = _real_multiplier(alpha[c], sx, sw[c], sr)
        assert 2 ** 30 <= abs(int(m0[c])) < 2 ** 31 and 1 <= sh[c] <= 62
        assert (m0[c] < 0) == (real < 0)
        approx = Fraction(int(m0[c]), 2 ** int(sh[c]))
        # nearest 31-bit mantissa to the fp64 value of the real multiplier (itself within 3 fp64
        # roundings of the exact one): relative error below 2^-31 + 2^-50
        assert abs(approx - real) <= abs(real) * (Fraction(1, 2 ** 31) + Fraction(1, 2 ** 50))


def test_multiplier_edge_cases(orc):
    z = np.zeros(1, np.int32)

    def one(a, sx=1.0, sw=1.0, sr=1.0):
        m0, sh, _, nsat = orc.fold_fixed_point(np.array([a], np.float32), None,
                                               np.array([sw], np.float32), None, z,
                                               np.float32(sx), 0, np.float32(sr))
        return int(m0[0]), int(sh[0]), nsat

    assert one(0.5) == (2 ** 30, 31, 0)                      # exact powers of two
    assert one(1.0) == (2 ** 30, 30, 0)
    assert one(-0.25) == (-2 ** 30, 32, 0)
    assert one(0.75) == (3 * 2 ** 29, 31, 0)
    # mantissa that rounds up to 2^31: (1 + 2^-23)(1 - 2^-23) = 1 - 2^-46 -> 2^30 * 2^-30
    assert one(1.0 + 2.0 ** -23, sx=1.0 - 2.0 ** -23) == (2 ** 30, 30, 0)
    # |M'| >= 2^30 is clamped and counted; 2^29 is still representable (shift 1)
    assert one(2.0 ** 29) == (2 ** 30, 1, 0)
    assert one(2.0 ** 30) == (2 ** 31 - 1, 1, 1)
    assert one(-3.0e9) == (-(2 ** 31 - 1), 1, 1)
    # smallest representable magnitude 2^-32 (shift 62); below it the channel maps to Z_r
    assert one(2.0 ** -32) == (2 ** 30, 62, 0)
    assert one(2.0 ** -33) == (0, 1, 0)
    assert one(1e-30) == (0, 1, 0)


def test_fixed_point_fold_offset_equals_float_fold_offset(orc):
    n = 256
    g = synth.normal(9002, 0, 5 * n).numpy()
    alpha = (1.0 + 0.2 * g[:n]).astype(np.float32)
    beta = (0.05 * g[n:2 * n]).astype(np.float32)
    sw = (np.abs(g[2 * n:3 * n]) * 1e-3 + 1e-4).astype(np.float32)
    bias = (0.02 * g[3 * n:4 * n]).astype(np.float32)
    colsum = np.rint(g[4 * n:] * 300).astype(np.int32)
    sx, zx, sr = np.float32(0.031), -7, np.float32(0.11)
    m0, sh, off, nsat = orc.fold_fixed_point(alpha, beta, sw, bias, colsum, sx, zx, sr)
    mult, off_f, nsat_f = orc.fold_int_offset(alpha, beta, sw, bias, colsum, sx, zx, sr)
    np.testing.assert_array_equal(off, off_f)
    assert nsat == nsat_f == 0
    # both multipliers are roundings of the same real number
    approx = m0.astype(np.float64) * np.exp2(-sh.astype(np.float64))
    assert np.max(np.abs(approx - mult.astype(np.float64)) / np.abs(approx)) <= 2.0 ** -24 + 2.0 ** -30


def test_fixed_point_epilogue_is_exact_round_half_up(orc):
    rows, n = 64, 48
    rs = np.random.RandomState(5)
    acc = rs.randint(-2 ** 31, 2 ** 31 - 1, size=(rows, n), dtype=np.int64).astype(np.int32)
    acc[:4] = rs.randint(-3000, 3000, size=(4, n))
    off = np.zeros(n, np.int32)
    m0 = (rs.randint(2 ** 30, 2 ** 31, size=n) * rs.choice([-1, 1], size=n)).astype(np.int32)
    sh = rs.randint(1, 63, size=n).astype(np.int32)
    sh[:8] = [62, 61, 1, 2, 31, 32, 33, 40]
    zr = 9
    out = orc.fixed_point_forward(acc, off, m0, sh, zr)
    for i in range(rows):
        for c in range(n):
            exact = Fraction(int(acc[i, c]) * int(m0[c]), 2 ** int(sh[c]))
            v = (int(acc[i, c]) * int(m0[c]) + 2 ** (int(sh[c]) - 1)) // 2 ** int(sh[c])
            assert abs(Fraction(v) - exact) <= Fraction(1, 2)
            if abs(Fraction(v) - exact) == Fraction(1, 2):
                assert Fraction(v) > exact                           # ties go up
            assert out[i, c] == min(127, max(-128, v + zr))
    # crafted ties: t * M0 / 2^shift = k + 1/2  ->  k + 1, for both signs of t
    t = np.array([[1, -1, 3, -3, 5, -5]], np.int32)
    out = orc.fixed_point_forward(t, np.zeros(6, np.int32), np.full(6, 2 ** 30, np.int32),
                                  np.full(6, 31, np.int32), 0)       # multiplier exactly 1/2
    np.testing.assert_array_equal(out[0], [1, 0, 2, -1, 3, -2])
    # the offset is added before the multiplication, in 64 bits (no int32 wrap)
    t = np.array([[2 ** 31 - 1]], np.int32)
    out = orc.fixed_point_forward(t, np.array([2 ** 30], np.int32), np.array([2 ** 30], np.int32),
                                  np.array([62], np.int32), 0)
    assert out[0, 0] == 1      # (2^31 - 1 + 2^30) * 2^-32 = 0.75 -> 1


def test_fixed_point_epilogue_against_float_epilogue(orc):
    """Same folded layer through both epilogues: at most one code apart, and only where the real
    value lies within the float path's rounding error of a tie."""
    rows, n, k = 96, 160, 256
    g = synth.normal(9003, 0, rows * k).numpy().reshape(rows, k)
    xq = np.clip(np.rint(g * 40), -128, 127).astype(np.int8)
    g = synth.normal(9003, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 40), -127, 127).astype(np.int8)
    acc = orc.gemm_i8(xq, wq)
    gg = synth.normal(9003, 2, 3 * n).numpy()
    alpha = (1.0 + 0.1 * gg[:n]).astype(np.float32)
    alpha[3] = -0.7                                         # a negative slope folds too
    beta = (0.3 * gg[n:2 * n]).astype(np.float32)
    sw = (np.abs(gg[2 * n:]) * 2e-3 + 5e-4).astype(np.float32)
    colsum = orc.colsum_i8(wq)
    sx, zx, sr, zr = np.float32(0.02), 11, np.float32(0.9), -4
    mult, off, _ = orc.fold_int_offset(alpha, beta, sw, None, colsum, sx, zx, sr)
    m0, sh, off2, _ = orc.fold_fixed_point(alpha, beta, sw, None, colsum, sx, zx, sr)
    np.testing.assert_array_equal(off, off2)
    r_float = orc.folded_forward(acc, off, mult, zr).astype(np.int32)
    r_fixed = orc.fixed_point_forward(acc, off, m0, sh, zr).astype(np.int32)
    diff = np.abs(r_float - r_fixed)
    assert diff.max() <= 1
    assert 0.1 < np.mean(np.abs(r_fixed) < 127), "codes should not all saturate"
    t = acc.astype(np.int64) + off.astype(np.int64)[None, :]
    for i, c in zip(*np.nonzero(diff)):
        real = Fraction(int(t[i, c])) * _real_multiplier(alpha[c], sx, sw[c], sr)
        frac = real - (real.numerator // real.denominator)
        assert abs(frac - Fraction(1, 2)) <= abs(real) * Fraction(1, 2 ** 22)
    assert np.mean(diff != 0) < 5e-3
