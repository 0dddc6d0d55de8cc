"""Pins for the oracle's quantized convolution (the integer product of Eq. 7 over a receptive
field; CWAC follows every quantized convolutional layer, Sec. 3.3, and folds into it, Sec. 3.4).
Expectations come from a hand-derived fixture, numpy sliding windows and the linear-layer
product, never from the function under test."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _windows_product(xq, wq, stride, pad, zx):
    """numpy: pad with the zero-point, gather windows, one integer tensordot."""
    b, h, w, c = xq.shape
    n, kh, kw, _ = wq.shape
    xp = np.full((b, h + 2 * pad, w + 2 * pad, c), zx, dtype=np.int64)
    xp[:, pad:pad + h, pad:pad + w, :] = xq
    win = np.lib.stride_tricks.sliding_window_view(xp, (kh, kw), axis=(1, 2))   # [b, H', W', c, kh, kw]
    win = win[:, ::stride, ::stride]
    out = np.einsum("bhwcij,nijc->bhwn", win, wq.astype(np.int64))
    return out.reshape(-1, n)


def test_worked_example(orc):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "conv_3x3_worked.txt"))
            if l.strip() and not l.startswith("#")]
    want = np.array(rows, dtype=np.int32).reshape(9, 1)
    x = np.arange(1, 10, dtype=np.int8).reshape(1, 3, 3, 1)
    w = np.array([[1, 0, -1], [2, 0, -2], [1, 0, -1]], dtype=np.int8).reshape(1, 3, 3, 1)
    np.testing.assert_array_equal(orc.conv2d_i8(x, w, stride=1, pad=1, zx=10), want)


@pytest.mark.parametrize("h,w,c,n,k,stride,pad,zx", [
    (7, 9, 16, 5, 3, 1, 1, -7), (8, 8, 16, 4, 3, 2, 1, 3), (9, 7, 32, 3, 1, 1, 0, 11),
    (11, 10, 16, 2, 7, 2, 3, -128), (6, 6, 16, 3, 3, 1, 0, 0), (5, 8, 16, 2, 1, 2, 0, 5)])
def test_against_numpy_windows(orc, h, w, c, n, k, stride, pad, zx):
    rng = np.random.default_rng(h * 100 + w)
    xq = rng.integers(-128, 128, (2, h, w, c), dtype=np.int64).astype(np.int8)
    wq = rng.integers(-127, 128, (n, k, k, c), dtype=np.int64).astype(np.int8)
    got = orc.conv2d_i8(xq, wq, stride, pad, zx)
    np.testing.assert_array_equal(got.astype(np.int64), _windows_product(xq, wq, stride, pad, zx))


def test_rectangular_filters(orc):
    """kh != kw: the two filter axes are not interchangeable."""
    rng = np.random.default_rng(8)
    xq = rng.integers(-128, 128, (2, 9, 10, 16), dtype=np.int64).astype(np.int8)
    for kh, kw, pad in [(1, 3, 0), (3, 1, 0), (5, 3, 1), (1, 7, 0)]:
        wq = rng.integers(-127, 128, (3, kh, kw, 16), dtype=np.int64).astype(np.int8)
        got = orc.conv2d_i8(xq, wq, 1, pad, 4)
        np.testing.assert_array_equal(got.astype(np.int64), _windows_product(xq, wq, 1, pad, 4))


def test_pointwise_convolution_is_the_linear_layer(orc):
    rng = np.random.default_rng(3)
    xq = rng.integers(-128, 128, (3, 5, 6, 32), dtype=np.int64).astype(np.int8)
    wq = rng.integers(-127, 128, (7, 1, 1, 32), dtype=np.int64).astype(np.int8)
    np.testing.assert_array_equal(orc.conv2d_i8(xq, wq), orc.gemm_i8(xq.reshape(-1, 32), wq.reshape(7, 32)))


def test_zero_point_term_with_padding(orc):
    """Eq. 6 <-> Eq. 7 for a padded convolution: sum w_q (x_q - Z_x) with real zeros outside the image
    equals acc - Z_x * sum(w_q), because the padding code is Z_x itself."""
    rng = np.random.default_rng(4)
    zx = -9
    xq = rng.integers(-128, 128, (1, 6, 5, 16), dtype=np.int64).astype(np.int8)
    wq = rng.integers(-127, 128, (4, 3, 3, 16), dtype=np.int64).astype(np.int8)
    acc = orc.conv2d_i8(xq, wq, 1, 1, zx).astype(np.int64)
    colsum = orc.colsum_i8(wq.reshape(4, -1)).astype(np.int64)
    centred = xq.astype(np.int64) - zx                    # real zero outside -> pad with 0
    want = _windows_product(centred, wq, 1, 1, 0)
    np.testing.assert_array_equal(acc - zx * colsum[None, :], want)
