"""Host-side check of the requantisation arithmetic the direct-to-LDS epilogue uses (Eq. 10's round, add Z_r,
clip): the output zero point rides in the constant of the rounding add.  The identity is emulated here in numpy
fp32 (round to nearest even, one rounding per operation, as on the device) for every int8 zero point and compared
with the oracle's plain definition on the same values - exact ties, saturation at both ends and 4-bit code ranges
included.  No GPU, no kernel code: it pins the algorithm the kernel encodes."""
import numpy as np
import pytest

F = np.float32
MAGIC = 12582912            # 1.5 * 2^23


def _codes_with_folded_zero_point(u, zr, qmin=-128, qmax=127):
    """What the epilogue computes from the fp32 value u = fl(acc * M') (already including the bias, if any)."""
    lo, hi = F(qmin - zr), F(qmax - zr)
    if zr % 2 == 0:
        c = F(MAGIC + zr)                                  # even constant: ties of the sum = ties of u
        s = (np.clip(u, lo, hi).astype(F) + c).astype(F)   # one fp32 add
        return (s.view(np.int32) & 0xff).astype(np.uint8).view(np.int8)
    # odd zero point: the chain runs on -u, the constant carries the even -zr - 1, the byte is complemented
    c = F(MAGIC - zr - 1)
    s = (np.clip(-u, -hi, -lo).astype(F) + c).astype(F)
    return ((~s.view(np.int32)) & 0xff).astype(np.uint8).view(np.int8)


def _values():
    rng = np.random.default_rng(11)
    grid = np.arange(-400, 400.25, 0.25, dtype=np.float64)             # every tie in range, and beyond both ends
    rand = rng.standard_normal(20000) * 90.0
    big = np.array([1e9, -1e9, 3e38, -3e38, 2.0 ** 23, -(2.0 ** 23), 1e-30, -1e-30, 0.0, -0.0])
    near = np.concatenate([np.nextafter(F(grid), F(np.inf)), np.nextafter(F(grid), F(-np.inf))]).astype(np.float64)
    return np.concatenate([grid, rand, big, near]).astype(F)


@pytest.mark.parametrize("qmin,qmax", [(-128, 127), (-8, 7), (-32, 31)])
def test_folded_zero_point_equals_round_then_add_then_clip(orc, qmin, qmax):
    u = _values()
    acc = np.arange(u.size, dtype=np.int32)[None, :] * 0 + 1       # acc = 1, offset = 0: u = 1 * mult = the value
    off = np.zeros(u.size, dtype=np.int32)
    for zr in range(qmin, qmax + 1):
        want = orc.folded_forward(acc, off, u, zr, qmin=qmin, qmax=qmax)[0]
        got = _codes_with_folded_zero_point(u, zr, qmin, qmax)
        # the definition itself, in numpy: clip(rint(u) + zr)
        plain = np.clip(np.rint(u.astype(np.float64)) + zr, qmin, qmax).astype(np.int8)
        np.testing.assert_array_equal(want, plain, err_msg=f"oracle vs definition, z_r = {zr}")
        np.testing.assert_array_equal(got, want, err_msg=f"folded constant vs oracle, z_r = {zr}")


def test_the_sum_stays_in_the_binade_of_unit_steps():
    """The trick needs clamp(u) + constant inside [2^23, 2^24): there fp32 steps are 1 and the low byte of the
    bit pattern is the low byte of the integer."""
    for zr in range(-128, 128):
        for n in (-128 - zr, 127 - zr):
            for c in (MAGIC + zr, MAGIC - zr - 1):
                for sgn in (1, -1):
                    assert 2 ** 23 <= c + sgn * n < 2 ** 24
