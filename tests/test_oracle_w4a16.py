"""Pins for the weight-only INT4 oracle (LLM setting of Sec. 4.4 with the CWAC
of Sec. 3.3-3.4).  Expectations come from numpy's own float16 type, exact
rational arithmetic, a hand-derived fixture and numpy matmul, never from the
oracle itself."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2505_20932_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def w4():
    from oracle import w4a16_oracle
    w4a16_oracle.build()
    return w4a16_oracle


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# ------------------------------------------------------------------ binary16
def test_f16_to_f32_all_patterns(w4):
    """Every one of the 65536 bit patterns against numpy's float16."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([w4.f16_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    np.testing.assert_array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f32_to_f16_against_numpy(w4):
    """Round-to-nearest-even incl. ties, subnormals, overflow, signed zero."""
    rng = np.random.default_rng(7)
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 70000.0, -65520.0, np.inf, -np.inf,
            2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 3 * 2.0 ** -25, 2.0 ** -26,
            2.0 ** -14 - 2.0 ** -25, 2.0 ** -14 - 2.0 ** -26, 1e-10, 1e-30]
    # exact midpoints between neighbouring binary16 numbers, both parities
    for b in (0x3c00, 0x3c01, 0x0400, 0x03ff, 0x0001, 0x7bfe, 0x2bcd, 0x5555):
        lo = np.array([b, b + 1], dtype=np.uint16).view(np.float16).astype(np.float64)
        vals += [float(lo.mean()), -float(lo.mean())]
    vals = np.array(vals, dtype=np.float32)
    rnd = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(3.0),
        (rng.standard_normal(5000) * 1e-6).astype(np.float32),
        (rng.standard_normal(5000) * 3e4).astype(np.float32),
        rng.integers(0, 2 ** 32, 20000, dtype=np.uint64).astype(np.uint32).view(np.float32)])
    rnd = rnd[~np.isnan(rnd)]
    x = np.concatenate([vals, rnd])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([w4.f32_to_f16(v) for v in x], dtype=np.uint16)
    np.testing.assert_array_equal(got, want)


# ------------------------------------------------------------------ quantizer
def test_group_quantizer_worked_example(w4):
    rows = _read_table("w4_group_unit_scale.txt")
    w = np.zeros((1, 128), dtype=np.float32)
    w[0, :len(rows)] = [float(r[0]) for r in rows]
    codes, scales, zeros = w4.quantize_groupwise(w)
    assert scales[0, 0] == np.float16(1.0) and zeros[0, 0] == 8
    np.testing.assert_array_equal(codes[0, :len(rows)], [int(r[1]) for r in rows])
    np.testing.assert_array_equal(codes[0, len(rows):], 8)
    wd = w4.dequant(codes, scales, zeros)
    np.testing.assert_array_equal(wd[0, :len(rows)], [float(r[2]) for r in rows])


def test_group_quantizer_against_exact_rational(w4):
    """Stored scale = correctly rounded binary16 of the fp32 quotient; zero-point and every code
    the nearest integers (within the fp32 division's rounding) with the stored scale."""
    w = (synth.normal(21, 1, 6 * 512).numpy() * 0.02 + 0.003).reshape(6, 512)
    w[2, 128:256] += 0.05           # a group that does not straddle zero: z clips at 0
    w[3, 0:128] -= 0.08             # all negative: z clips at 15
    codes, scales, zeros = w4.quantize_groupwise(w)
    assert codes.max() <= 15 and zeros.max() <= 15
    for r in range(6):
        for g in range(4):
            grp = w[r, g * 128:(g + 1) * 128]
            mn, mx = grp.min(), grp.max()
            s32 = np.float32(np.float32(mx - mn) / np.float32(15.0))
            assert scales[r, g] == np.float16(s32)                 # numpy's own rounding
            s = Fraction(float(scales[r, g]))
            zr = Fraction(-float(mn)) / s
            z = int(zeros[r, g])
            assert z == min(15, max(0, round(zr))) or abs(zr - z) <= Fraction(1, 2) + Fraction(1, 10 ** 6)
            for i in range(128):
                t = Fraction(float(grp[i])) / s
                c = int(codes[r, g * 128 + i])
                ideal = t + z
                if ideal <= 0:
                    assert c == 0 or abs(ideal - c) <= Fraction(1, 2) + Fraction(1, 10 ** 5)
                elif ideal >= 15:
                    assert c == 15 or abs(ideal - c) <= Fraction(1, 2) + Fraction(1, 10 ** 5)
                else:
                    assert abs(ideal - c) <= Fraction(1, 2) + Fraction(1, 10 ** 5)
    assert zeros[2, 1] == 0 and zeros[3, 0] == 15
    # group extremes reach (or clip at) the end codes where the group straddles zero
    assert codes[0, :128].min() == 0 and codes[0, :128].max() == 15


def test_group_quantizer_degenerate_groups(w4):
    w = np.zeros((2, 256), dtype=np.float32)
    w[0, :128] = 0.25                   # constant group: scale floored, every weight the same code
    w[1, :128] = np.linspace(-1e4, 1e4, 128, dtype=np.float32)
    w[1, 128:] = np.linspace(-1e6, 1e6, 128, dtype=np.float32)   # scale beyond the binary16 range
    codes, scales, zeros = w4.quantize_groupwise(w)
    assert scales[0, 0] == np.float16(2.0 ** -14)
    assert len(set(codes[0, :128].tolist())) == 1
    assert scales[1, 1] == np.float16(65504.0)                   # largest finite value, never inf
    wd = w4.dequant(codes, scales, zeros)
    assert np.isfinite(wd[:, :128]).all() and np.isfinite(wd[0]).all()


def test_round_trip_error(w4):
    """|w - Wd| <= s/2 (+ the binary16 rounding of the product) for weights inside the grid."""
    w = (synth.normal(22, 1, 8 * 1024).numpy() * 0.02).reshape(8, 1024)
    codes, scales, zeros = w4.quantize_groupwise(w)
    wd = w4.dequant(codes, scales, zeros)
    s = np.repeat(scales.astype(np.float64), 128, axis=1)
    z = np.repeat(zeros.astype(np.float64), 128, axis=1)
    inside = (w / s + z >= 0) & (w / s + z <= 15)
    err = np.abs(w.astype(np.float64) - wd)
    bound = s / 2 + np.abs(wd) * 2.0 ** -11 + 1e-9
    assert (err[inside] <= bound[inside]).all()
    # outside the grid only by the rounding of the zero-point: at most one step
    assert (err[~inside] <= 1.5 * s[~inside]).all()


def test_dequant_against_numpy_float16(w4):
    """Wd = RN16(s * (c - z)): numpy multiplies float16 scalars with a single rounding."""
    rng = np.random.default_rng(3)
    n, k = 16, 512
    codes = rng.integers(0, 16, (n, k), dtype=np.uint8)
    zeros = rng.integers(0, 16, (n, k // 128), dtype=np.uint8)
    scales = (rng.random((n, k // 128)) * 0.01 + 1e-4).astype(np.float16)
    scales[0, 0] = np.float16(2.0 ** -14)       # products below 2^-14 * 1 are exact, above stay normal
    scales[1, 1] = np.float16(6e-8)             # subnormal scale: subnormal products are kept
    scales[2, 2] = np.float16(3000.0)
    wd = w4.dequant(codes, scales, zeros)
    d = (codes.astype(np.int32) - np.repeat(zeros.astype(np.int32), 128, axis=1)).astype(np.float16)
    want = (np.repeat(scales, 128, axis=1) * d).astype(np.float32)
    np.testing.assert_array_equal(wd, want)
    # and against exact rational arithmetic on a sample
    for (r, c) in [(0, 5), (1, 130), (2, 300), (7, 77), (15, 511)]:
        exact = Fraction(float(scales[r, c // 128])) * (int(codes[r, c]) - int(zeros[r, c // 128]))
        got = Fraction(float(wd[r, c]))
        if exact != 0 and abs(exact) >= Fraction(1, 2 ** 14):
            assert abs(got - exact) <= abs(exact) * Fraction(1, 2 ** 11)
        else:
            assert abs(got - exact) <= Fraction(1, 2 ** 25)


# ------------------------------------------------------------------ product, compensation
def test_product_against_numpy(w4):
    rng = np.random.default_rng(5)
    m, n, k = 37, 24, 256
    x16 = rng.standard_normal((m, k)).astype(np.float16)
    wd = (rng.standard_normal((n, k)) * 0.02).astype(np.float16).astype(np.float32)
    acc, mag = w4.product(x16, wd)
    want = x16.astype(np.float64) @ wd.astype(np.float64).T
    np.testing.assert_allclose(acc, want, rtol=0, atol=1e-12)
    wantm = np.abs(x16.astype(np.float64)) @ np.abs(wd.astype(np.float64)).T
    np.testing.assert_allclose(mag, wantm, rtol=1e-13)
    rows = np.array([36, 0, 5], dtype=np.int64)
    acc_r, _ = w4.product(x16, wd, rows)
    np.testing.assert_array_equal(acc_r, acc[rows])
    # not symmetric in its operands: a transposed weight matrix is a different product
    x2 = np.zeros((2, 128), dtype=np.float16)
    x2[0, 3] = 1.0
    x2[1, 9] = 2.0
    w2 = np.zeros((3, 128), dtype=np.float32)
    w2[2, 3] = 5.0
    w2[1, 9] = -4.0
    a2, _ = w4.product(x2, w2)
    np.testing.assert_array_equal(a2, [[0, 0, 5], [0, -8, 0]])


def test_fold_against_exact_rational(w4):
    rng = np.random.default_rng(9)
    n = 64
    alpha = (1 + 0.1 * rng.standard_normal(n)).astype(np.float32)
    beta = (0.05 * rng.standard_normal(n)).astype(np.float32)
    bias = (0.02 * rng.standard_normal(n)).astype(np.float32)
    mult, fbias = w4.fold(alpha, beta, bias, n)
    np.testing.assert_array_equal(mult, alpha)
    for c in range(n):
        exact = Fraction(float(alpha[c])) * Fraction(float(bias[c])) + Fraction(float(beta[c]))
        ulp = Fraction(float(np.spacing(np.abs(fbias[c]))))
        assert abs(Fraction(float(fbias[c])) - exact) <= ulp / 2 + Fraction(1, 10 ** 20)
    # no compensation: multiplier one, constant = layer bias; no bias either: zero
    m1, f1 = w4.fold(None, None, bias, n)
    np.testing.assert_array_equal(m1, np.ones(n, np.float32))
    np.testing.assert_array_equal(f1, bias)
    m0, f0 = w4.fold(None, None, None, n)
    assert (m0 == 1).all() and (f0 == 0).all()
    mi, fi = w4.fold(np.ones(n, np.float32), np.zeros(n, np.float32), bias, n)
    np.testing.assert_array_equal(mi, m1)
    np.testing.assert_array_equal(fi, f1)


def test_folded_equals_unfolded(w4):
    """alpha*(y + b) + beta == y*alpha + (alpha*b + beta): the fold changes the real value only by
    the fp32 rounding of the constant."""
    rng = np.random.default_rng(10)
    rows, n = 50, 32
    acc = rng.standard_normal((rows, n)) * 3
    alpha = (1 + 0.2 * rng.standard_normal(n)).astype(np.float32)
    alpha[3] = -0.5
    beta = (0.1 * rng.standard_normal(n)).astype(np.float32)
    bias = (0.02 * rng.standard_normal(n)).astype(np.float32)
    unf = w4.unfolded(acc, bias, alpha, beta)
    want = alpha.astype(np.float64) * (acc + bias.astype(np.float64)) + beta.astype(np.float64)
    np.testing.assert_allclose(unf, want, rtol=1e-15, atol=1e-15)
    mult, fbias = w4.fold(alpha, beta, bias, n)
    fol = w4.folded_real(acc, mult, fbias)
    gap = np.abs(fol - unf)
    assert (gap <= np.spacing(np.abs(fbias)).astype(np.float64)[None, :] / 2 + 1e-15).all()
    # argument order guard: alpha multiplies, beta adds
    one = w4.unfolded(np.ones((1, 2)), None, np.array([2, 3], np.float32), np.array([10, 20], np.float32))
    np.testing.assert_array_equal(one, [[12, 23]])


def test_epilogue_f32_fixed_order(w4):
    """u = fl(fl(acc * mult) + fbias), then RN16: checked with numpy float32 scalars."""
    rng = np.random.default_rng(11)
    acc = (rng.standard_normal((9, 16)) * 100).astype(np.float32)
    mult = (1 + 0.3 * rng.standard_normal(16)).astype(np.float32)
    fbias = rng.standard_normal(16).astype(np.float32)
    o32, o16 = w4.epilogue_f32(acc, mult, fbias)
    want = (acc * mult[None, :]).astype(np.float32) + fbias[None, :]
    np.testing.assert_array_equal(o32, want.astype(np.float32))
    np.testing.assert_array_equal(o16.view(np.uint16), want.astype(np.float16).view(np.uint16))


def test_compensation_reduces_calibration_error(w4, orc):
    """End to end on a small LLM-shaped layer: the closed-form fit (Eq. 4-5) on the weight-only
    layer's outputs never increases the calibration error of any channel."""
    n, k, rows = 48, 512, 600
    w = (synth.normal(31, 1, n * k).numpy() * 0.02).reshape(n, k)
    x = synth.normal(31, 2, rows * k).numpy().reshape(rows, k)
    x[:, 7] *= 60.0
    x16 = x.astype(np.float16)
    codes, scales, zeros = w4.quantize_groupwise(w)
    wd = w4.dequant(codes, scales, zeros)
    acc, _ = w4.product(x16, wd)
    y_full = (x16.astype(np.float64) @ w.astype(np.float64).T).astype(np.float32)
    y_quant = acc.astype(np.float32)
    alpha, beta = orc.fit(y_full, y_quant)[:2]
    mult, fbias = w4.fold(alpha, beta, None, n)
    yc = w4.folded_real(acc, mult, fbias)
    e0 = ((y_quant.astype(np.float64) - y_full) ** 2).sum(axis=0)
    e1 = ((yc - y_full) ** 2).sum(axis=0)
    assert (e1 <= e0 * (1 + 1e-6)).all()
    assert e1.sum() < e0.sum()
