"""Pins for the oracle's quantizers (Sec. 3.2, Eq. 1-2) and integer product
(Sec. 3.4, Eq. 6-7).  Expectations come from a hand-derived fixture, exact
rational arithmetic and numpy integer matmul, never from the oracle itself."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2505_20932_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_unit_scale_worked_example(orc):
    """Hand-derived example: s = 1, z = 64, ties go to even."""
    rows = _read_table("quantizer_unit_scale.txt")
    x = np.array([float(r[0]) for r in rows], dtype=np.float32)
    want = np.array([int(r[1]) for r in rows], dtype=np.int32)
    s, z = orc.qparams_asym(-64.0, 191.0, 8)
    assert s == np.float32(1.0) and z == 64
    got = orc.quantize_asym(x, s, z, 8)
    np.testing.assert_array_equal(got, want)
    # signed storage is a relabelling by 128 of code and zero-point
    q8 = orc.quantize_act_i8(x, s, z - 128)
    np.testing.assert_array_equal(q8.astype(np.int32) + 128, want)


@pytest.mark.parametrize("bits", [4, 6, 8])
def test_eq2_against_exact_rational(orc, bits):
    """s is the correctly rounded quotient; z the nearest integer to -min/s."""
    x = synth.normal(11, bits, 4096).numpy() * 3.0 + 0.7
    mn, mx = orc.range_f32(x)
    assert mn == x.min() and mx == x.max()
    s, z = orc.qparams_asym(mn, mx, bits)
    levels = (1 << bits) - 1
    diff = Fraction(float(np.float32(mx) - np.float32(mn)))      # fp32 subtraction, as Eq. 2 in fp32
    exact = diff / levels
    # correctly rounded fp32 division: the result is within half an ulp of the exact quotient
    ulp = Fraction(float(np.spacing(np.float32(s))))
    assert abs(Fraction(float(s)) - exact) <= ulp / 2
    zr = Fraction(-float(mn)) / Fraction(float(s))
    assert abs(zr - z) <= Fraction(1, 2) + Fraction(1, 1000)
    assert 0 <= z <= levels


@pytest.mark.parametrize("bits", [4, 8])
def test_eq1_round_trip_and_endpoints(orc, bits):
    x = synth.normal(12, bits, 20000).numpy() * 2.0 - 0.3
    mn, mx = orc.range_f32(x)
    s, z = orc.qparams_asym(mn, mx, bits)
    q = orc.quantize_asym(x, s, z, bits)
    levels = (1 << bits) - 1
    assert q.min() == 0 and q.max() == levels          # min -> code 0, max -> top code
    assert q[np.argmin(x)] == 0 and q[np.argmax(x)] == levels
    # in-range values are reproduced to within half a step (plus fp32 slack)
    deq = np.float64(s) * (q.astype(np.float64) - z)
    assert np.max(np.abs(deq - x.astype(np.float64))) <= 0.5 * float(s) * (1 + 1e-4) + 1e-6
    # each code is the nearest integer to x/s + z (exact rationals, sampled)
    for i in range(0, x.size, 997):
        v = Fraction(float(x[i])) / Fraction(float(s)) + z
        if 0 < v < levels:
            assert abs(v - int(q[i])) <= Fraction(1, 2) + Fraction(1, 1000)
    # values far outside the range clip to the end codes
    far = np.array([mn - 100.0, mx + 100.0, -np.inf, np.inf], dtype=np.float32)
    np.testing.assert_array_equal(orc.quantize_asym(far, s, z, bits), [0, levels, 0, levels])


def test_rows_sym(orc):
    w = synth.normal(13, 0, 37 * 129).numpy().reshape(37, 129) * 0.02
    w[5, :] = 0.0                                      # degenerate all-zero row
    q, s = orc.quantize_rows_sym(w)
    amax = np.abs(w).max(axis=1)
    for r in range(37):
        if r == 5:
            assert np.all(q[r] == 0) and s[r] > 0
            continue
        ulp = Fraction(float(np.spacing(np.float32(s[r]))))
        assert abs(Fraction(float(s[r])) - Fraction(float(amax[r])) / 127) <= ulp / 2
        assert np.abs(q[r]).max() == 127               # the extreme element maps to +-127
        assert q[r].min() >= -127                      # symmetric range, -128 unused
        err = np.abs(np.float64(s[r]) * q[r] - w[r].astype(np.float64))
        assert err.max() <= 0.5 * float(s[r]) * (1 + 1e-4)
    # sign symmetry: Q(-w) = -Q(w), same scales
    q2, s2 = orc.quantize_rows_sym(-w)
    np.testing.assert_array_equal(q2, -q)
    np.testing.assert_array_equal(s2, s)


def _rand_i8(seed, shape, lo=-128, hi=127):
    z = synth.normal(seed, 0, int(np.prod(shape))).numpy().reshape(shape)
    return np.clip(np.rint(z * 50.0), lo, hi).astype(np.int8)


def test_gemm_against_numpy(orc):
    xq = _rand_i8(21, (23, 96))
    wq = _rand_i8(22, (17, 96), -127, 127)
    xq[0, :] = -128
    wq[0, :] = 127                                     # extreme products
    want = xq.astype(np.int64) @ wq.astype(np.int64).T
    got = orc.gemm_i8(xq, wq)
    assert got.dtype == np.int32 and got.shape == (23, 17)
    np.testing.assert_array_equal(got.astype(np.int64), want)
    rows = np.array([22, 0, 7, 7], dtype=np.int64)
    np.testing.assert_array_equal(orc.gemm_i8(xq, wq, rows=rows).astype(np.int64), want[rows])
    np.testing.assert_array_equal(orc.colsum_i8(wq).astype(np.int64),
                                  wq.astype(np.int64).sum(axis=1))
    # a transposed-operand mistake would show here: x [m,k] and w [n,k] are not interchangeable
    assert not np.array_equal(want, (wq.astype(np.int64)[:, :23] @ xq.astype(np.int64)[:17, :23].T).T)


def test_eq6_equals_eq7(orc):
    """The product of zero-point-shifted codes (Eq. 6) equals the four-term
    expansion that the engine evaluates (Eq. 7), also with weight zero-points."""
    xq = _rand_i8(31, (9, 64))
    wq = _rand_i8(32, (11, 64))
    zw = np.array([0, 3, -7, 100, -128, 127, 1, 0, -1, 5, 9], dtype=np.int32)
    for zx in (0, -128, 17, 127):
        direct = orc.product_zp_direct(xq, wq, zx, zw)
        expanded = orc.product_zp_expanded(xq, wq, zx, zw)
        want = (xq.astype(np.int64) - zx) @ (wq.astype(np.int64) - zw[:, None]).T
        np.testing.assert_array_equal(direct, want)
        np.testing.assert_array_equal(expanded, want)
    # symmetric weights (Z_W = 0): only the Z_x * colsum correction survives
    zx = -23
    acc = orc.gemm_i8(xq, wq).astype(np.int64)
    cs = orc.colsum_i8(wq).astype(np.int64)
    np.testing.assert_array_equal(acc - zx * cs[None, :],
                                  orc.product_zp_direct(xq, wq, zx, np.zeros(11, np.int32)))
