"""Pins for the oracle's CWAC fit (Sec. 3.3, Eq. 3-5): brute-force least
squares, library routines, planted models, invariants."""
import os

import numpy as np
import pytest

from paper_2505_20932_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _pair(seed, rows, c, noise=0.05):
    yq = synth.normal(seed, 0, rows * c).numpy().reshape(rows, c).astype(np.float32)
    e = synth.normal(seed, 1, rows * c).numpy().reshape(rows, c)
    gain = 1.0 + 0.2 * synth.normal(seed, 2, c).numpy()
    shift = 0.3 * synth.normal(seed, 3, c).numpy()
    yf = (gain[None, :] * yq + shift[None, :] + noise * e).astype(np.float32)
    return yf, yq


def test_moments_against_numpy(orc):
    yf, yq = _pair(41, 301, 13)
    mom = orc.channel_moments(yf, yq)
    f64, q64 = yf.astype(np.float64), yq.astype(np.float64)
    np.testing.assert_allclose(mom[0], f64.mean(0), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(mom[1], q64.mean(0), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(mom[2], q64.var(0), rtol=1e-12)
    np.testing.assert_allclose(mom[4], f64.var(0), rtol=1e-12)
    for c in range(13):
        cov = np.cov(q64[:, c], f64[:, c], bias=True)[0, 1]
        assert abs(mom[3][c] - cov) <= 1e-12 * abs(cov) + 1e-15


def test_fit_is_the_least_squares_minimiser(orc):
    """Eq. 4-5 must equal a brute-force 2-parameter least-squares solve (Eq. 3)."""
    yf, yq = _pair(42, 64, 8, noise=0.3)
    alpha, beta = orc.fit(yf, yq)
    for c in range(8):
        a_mat = np.stack([yq[:, c].astype(np.float64), np.ones(64)], axis=1)
        sol, *_ = np.linalg.lstsq(a_mat, yf[:, c].astype(np.float64), rcond=None)
        assert abs(alpha[c] - sol[0]) <= 1e-6 * max(1.0, abs(sol[0]))
        assert abs(beta[c] - sol[1]) <= 1e-6 * max(1.0, abs(sol[1]))
        p = np.polyfit(yq[:, c].astype(np.float64), yf[:, c].astype(np.float64), 1)
        assert abs(alpha[c] - p[0]) <= 1e-6 and abs(beta[c] - p[1]) <= 1e-6
        # grid search around the solution never finds a smaller residual
        def loss(a, b):
            r = yf[:, c].astype(np.float64) - (a * yq[:, c].astype(np.float64) + b)
            return float(r @ r)
        base = loss(float(alpha[c]), float(beta[c]))
        for da in (-1e-3, 1e-3):
            for db in (-1e-3, 1e-3):
                assert loss(float(alpha[c]) + da, float(beta[c]) + db) > base


def test_planted_and_identity(orc):
    yq = synth.normal(43, 0, 500 * 6).numpy().reshape(500, 6).astype(np.float32)
    a = np.array([0.5, 1.0, 2.0, -1.5, 1.25, 0.75], dtype=np.float32)   # exact in fp32
    d = np.array([0.0, 1.0, -2.0, 0.5, 8.0, -0.25], dtype=np.float32)
    yf = (a[None, :].astype(np.float64) * yq + d[None, :]).astype(np.float32)
    alpha, beta = orc.fit(yf, yq)
    np.testing.assert_allclose(alpha, a, rtol=2e-6)
    np.testing.assert_allclose(beta, d, rtol=2e-6, atol=2e-6)
    alpha, beta = orc.fit(yq, yq)                     # Y_quant == Y_full
    np.testing.assert_array_equal(alpha, np.ones(6, np.float32))
    np.testing.assert_allclose(beta, 0.0, atol=1e-7)


def test_residual_orthogonality_and_equivariance(orc):
    yf, yq = _pair(44, 777, 5, noise=0.5)
    alpha, beta = orc.fit(yf, yq)
    res = yf.astype(np.float64) - (alpha.astype(np.float64) * yq + beta.astype(np.float64))
    scale = np.abs(yf).sum(0)
    assert np.all(np.abs(res.sum(0)) <= 1e-5 * scale)                  # residual _|_ 1
    assert np.all(np.abs((res * yq).sum(0)) <= 1e-5 * scale * np.abs(yq).max())  # residual _|_ Y_quant
    # Y_quant -> k Y_quant + h  =>  alpha -> alpha / k, beta -> beta - alpha h / k  (k, h exact in fp32)
    k, h = 4.0, 0.5
    yq2 = (k * yq + h).astype(np.float32)
    a2, b2 = orc.fit(yf, yq2)
    np.testing.assert_allclose(a2, alpha / k, rtol=1e-5)
    np.testing.assert_allclose(b2, beta - alpha * h / k, rtol=1e-5, atol=1e-6)
    # swapping the roles of full and quant is a different regression (guards argument order)
    a3, _ = orc.fit(yq, yf)
    assert np.max(np.abs(a3 - alpha)) > 1e-3


def test_large_mean_channels_are_stable(orc):
    """|mean| >> std: a one-pass E[xy]-E[x]E[y] in low precision would fail here."""
    yq = (synth.normal(45, 0, 4000 * 3).numpy().reshape(4000, 3) * 0.01 + 1000.0).astype(np.float32)
    e = synth.normal(45, 1, 4000 * 3).numpy().reshape(4000, 3)
    yf = (yq.astype(np.float64) + 0.001 * e).astype(np.float32)
    alpha, beta = orc.fit(yf, yq)
    for c in range(3):
        p = np.polyfit(yq[:, c].astype(np.float64) - 1000.0, yf[:, c].astype(np.float64), 1)
        assert abs(alpha[c] - p[0]) <= 1e-6 * abs(p[0])


def test_degenerate_channels(orc):
    yf, yq = _pair(46, 50, 4)
    yq[:, 1] = 3.0                                      # constant quantized channel
    yf[:, 2] = 0.25                                     # constant full-precision channel: covariance exactly 0
    yq[:, 3] = 0.0                                      # constant at zero
    mom = orc.channel_moments(yf, yq)
    alpha, beta, ndeg = orc.solve(mom)
    assert ndeg == 3
    assert alpha[1] == 1.0 and alpha[2] == 1.0 and alpha[3] == 1.0
    assert beta[2] == np.float32(0.25 - mom[1][2])
    assert beta[1] == np.float32(mom[0][1] - 3.0)
    assert beta[3] == np.float32(mom[0][3])
    assert np.all(np.isfinite(alpha)) and np.all(np.isfinite(beta))
    # an exactly zero slope cannot be folded (Eq. 10 divides by alpha): shift-only fallback
    mom2 = mom.copy()
    mom2[3][0] = 0.0
    a2, b2, nd2 = orc.solve(mom2)
    assert nd2 == 4 and a2[0] == 1.0 and b2[0] == np.float32(mom[0][0] - mom[1][0])


def test_parameter_count_matches_printed_delta(orc):
    """Two 32-bit parameters per output channel of every linear reproduce the
    extra-storage column of the paper's ImageNet tables."""
    wl = synth.WORKLOADS[3]
    per_block = sum(l.n for l in wl.layers[:4])
    with open(os.path.join(GOLDEN, "cwac_delta_mb.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert per_block == int(rows[0][2])                # ViT-B block: 2304 + 768 + 3072 + 768
    yf, yq = _pair(47, 40, 16)
    alpha, beta = orc.fit(yf, yq)
    assert alpha.shape == beta.shape == (16,) and alpha.dtype == np.float32
    bytes_per_channel = alpha.itemsize + 4             # fp32 gain + 32-bit offset
    for _, blocks, chans, printed in rows:
        mb = int(blocks) * int(chans) * bytes_per_channel / 1e6
        assert round(mb, 1) == float(printed), (mb, printed)


def test_fit_error_shrinks_with_the_calibration_set(orc):
    """Synthetic analogue of the paper's calibration-set-size ablation (Sec. 4.5): for
    Y_full = a * Y_quant + d + noise the closed-form estimate approaches (a, d) like 1/sqrt(N),
    the textbook rate of a least-squares slope."""
    c = 64
    a = (0.8 + 0.4 * np.abs(synth.normal(55, 0, c).numpy())).astype(np.float64)
    d = synth.normal(55, 1, c).numpy().astype(np.float64) * 0.3
    errs = []
    for n_rows in (32, 128, 512, 2048, 8192):
        yq = synth.normal(56, n_rows, n_rows * c).numpy().reshape(n_rows, c).astype(np.float32)
        noise = synth.normal(57, n_rows, n_rows * c).numpy().reshape(n_rows, c) * 0.1
        yf = (a[None, :] * yq + d[None, :] + noise).astype(np.float32)
        alpha, beta = orc.fit(yf, yq)
        errs.append(float(np.sqrt(np.mean((alpha - a) ** 2 + (beta - d) ** 2))))
    # every 4x in rows roughly halves the error; 256x in rows: 16x, within a factor of 2
    assert all(e1 < 0.8 * e0 for e0, e1 in zip(errs, errs[1:])), errs
    assert 8.0 < errs[0] / errs[-1] < 32.0, errs
    # standard error of the slope: sigma_noise / (sigma_q * sqrt(N)); of the intercept about the same
    assert errs[-1] < 3.0 * 0.1 * np.sqrt(2.0 / 8192)
