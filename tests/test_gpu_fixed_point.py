"""GPU parity of the integer-only engine form: cwac_fold_fixed_point and
qlinear_cwac_forward_fixed_point against the oracle, bit for bit (integer work), on every kernel
and tile shape, edge tiles, extreme multipliers and shifts; at a full layer size on sampled rows."""

import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth
from tuning import tuning_of

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def _fold_inputs(seed, n):
    g = synth.normal(seed, 0, 5 * n).numpy()
    alpha = (1.0 + 0.2 * g[:n]).astype(np.float32)
    alpha[1 % n] = -0.6
    beta = (0.05 * g[n:2 * n]).astype(np.float32)
    sw = (np.abs(g[2 * n:3 * n]) * 1e-3 + 1e-4).astype(np.float32)
    bias = (0.02 * g[3 * n:4 * n]).astype(np.float32)
    colsum = np.rint(g[4 * n:] * 300).astype(np.int32)
    return alpha, beta, sw, bias, colsum


def test_fold_fixed_point_bit_exact(orc):
    n = 1000
    alpha, beta, sw, bias, colsum = _fold_inputs(8101, n)
    # extreme multipliers: clamped, vanishing, exact powers of two, the carry case
    alpha[10], sw[10] = 3.0e9, 1.0
    alpha[11], sw[11] = 1e-30, 1.0
    alpha[12], sw[12] = 0.5, 1.0
    alpha[13], sw[13] = 2.0 ** -32, 1.0
    sx, zx, sr = np.float32(1.0), -7, np.float32(1.0)
    for with_fit, with_bias in ((True, True), (False, True), (True, False)):
        a, b = (alpha, beta) if with_fit else (None, None)
        bi = bias if with_bias else None
        m0_0, sh_0, off_0, nsat_0 = orc.fold_fixed_point(a, b, sw, bi, colsum, sx, zx, sr)
        qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, float(sx), zx, float(sr), 0)
        m0 = torch.empty(n, dtype=torch.int32, device=DEV)
        sh = torch.empty(n, dtype=torch.int32, device=DEV)
        off = torch.empty(n, dtype=torch.int32, device=DEV)
        nsat = torch.full((1,), -5, dtype=torch.int32, device=DEV)
        P.cwac_fold_fixed_point(dev(a), dev(b), dev(sw), dev(bi), dev(colsum), qp, m0, sh, off, nsat)
        np.testing.assert_array_equal(host(m0), m0_0)
        np.testing.assert_array_equal(host(sh), sh_0)
        np.testing.assert_array_equal(host(off), off_0)
        assert int(host(nsat)[0]) == nsat_0
    assert nsat_0 >= 1
    # realistic scales too (sx, sr not 1)
    sx, sr = np.float32(0.031), np.float32(0.11)
    m0_0, sh_0, off_0, _ = orc.fold_fixed_point(alpha, beta, sw, bias, colsum, sx, zx, sr)
    qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, float(sx), zx, float(sr), 0)
    P.cwac_fold_fixed_point(dev(alpha), dev(beta), dev(sw), dev(bias), dev(colsum), qp, m0, sh, off)
    np.testing.assert_array_equal(host(m0), m0_0)
    np.testing.assert_array_equal(host(sh), sh_0)
    np.testing.assert_array_equal(host(off), off_0)
    with pytest.raises(P.CwacError):                      # per-token scales have no integer form
        P.cwac_fold_fixed_point(dev(alpha), dev(beta), dev(sw), None, dev(colsum),
                                P.make_qparams(P.CWAC_EPI_FP_BIAS, True, 1.0, 0, 1.0, 0), m0, sh, off)


def _forward(xq, wq, qp, m0, sh, off, tile=None, ldo=None, wgs=0):
    m, n = xq.shape[0], wq.shape[0]
    if ldo is None:
        out = torch.empty(m, n, dtype=torch.int8, device=DEV)
        view = out
    else:
        out = torch.full((m, ldo), 77, dtype=torch.int8, device=DEV)
        view = out[:, :n]
    P.qlinear_cwac_forward_fixed_point(dev(xq), dev(wq), qp, dev(m0), dev(sh), dev(off), view,
                                       tuning=tuning_of(tile, pipe="persist" if wgs else None,
                                                        persist_workgroups=wgs))
    return host(out)


@pytest.mark.parametrize("m,n,k,tile", [
    (197, 1152, 384, 64), (197, 1152, 384, 128), (197, 1152, 384, 256),
    (77, 50, 48, 64), (131, 203, 112, 128),
    (256, 256, 128, "fast"), (300, 520, 384, "fast"), (700, 1030, 1152, "fast"),
])
def test_forward_fixed_point_bit_exact(orc, m, n, k, tile):
    print(f"fixed-point forward {m} x {n} x {k} tile={tile}", flush=True)
    g = synth.normal(8200 + m, 0, m * k).numpy().reshape(m, k)
    xq = np.clip(np.rint(g * 60), -128, 127).astype(np.int8)
    g = synth.normal(8200 + m, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 60), -127, 127).astype(np.int8)
    acc = orc.gemm_i8(xq, wq)
    rs = np.random.RandomState(m)
    # multipliers sized so that codes spread over the int8 range; a few extreme channels
    scale = 40.0 / (3600.0 * np.sqrt(k))
    real = scale * np.exp(0.3 * synth.normal(8200 + m, 2, n).numpy()) * rs.choice([-1.0, 1.0], size=n)
    mant, e = np.frexp(np.abs(real))
    m0 = (np.rint(mant * 2.0 ** 31) * np.sign(real)).astype(np.int64)
    sh = (31 - e).astype(np.int32)
    carry = np.abs(m0) == 2 ** 31
    m0[carry] //= 2
    sh[carry] -= 1
    m0 = m0.astype(np.int32)
    m0[0], sh[0] = 2 ** 31 - 1, 1             # huge multiplier: every non-zero t saturates
    m0[1], sh[1] = -(2 ** 30), 62             # vanishing multiplier
    m0[2], sh[2] = 0, 1
    m0[3], sh[3] = 2 ** 30, 31                # exactly 1/2: ties on every odd t
    off = np.rint(synth.normal(8200 + m, 3, n).numpy() * 500).astype(np.int32)
    for zr, (qmin, qmax) in ((5, (-128, 127)), (-3, (-8, 7))):
        qp = P.make_qparams(z_r=zr, qmin=qmin, qmax=qmax)
        want = orc.fixed_point_forward(acc, off, m0, sh, zr, qmin, qmax)
        for ldo in (None, n + 5):
            got = _forward(xq, wq, qp, m0, sh, off, tile=tile, ldo=ldo)
            np.testing.assert_array_equal(got[:, :n], want)
            if ldo:
                assert np.all(got[:, n:] == 77)
        if tile == "fast" and k % 128 == 0:
            # persistent workgroups that walk several tiles each (the multiplier and shift of the next tile are
            # fetched under a tile's epilogue), with and without a split last round
            for wgs in (1, 2, 3):
                np.testing.assert_array_equal(_forward(xq, wq, qp, m0, sh, off, tile=tile, wgs=wgs), want)
    assert 0.05 < np.mean(np.abs(want.astype(np.int32)) < 7)


def test_forward_fixed_point_full_size(orc):
    """Config 2's layer at its full size in the automatic launch configuration: the whole
    integer-only pipeline (fold -> forward) on sampled rows, and next to the fp32 epilogue."""
    wl = synth.WORKLOADS[2]
    ly = wl.layers[0]
    m, n, k = wl.m, ly.n, ly.k
    w_t, b_t = synth.weights(wl, 0)
    x_t = synth.activations(wl, 0, m)
    rows = np.unique(np.concatenate([np.arange(0, 8), np.arange(250, 262), np.arange(m - 8, m),
                                     np.arange(300, m - 300, (m - 600) // 20)]))
    seed = wl.seed(0) + 55
    alpha = (1.0 + 0.05 * synth.normal(seed, 0, n).numpy()).astype(np.float32)
    beta = (0.02 * synth.normal(seed, 1, n).numpy()).astype(np.float32)
    w, x, bias = w_t.numpy(), x_t.numpy(), b_t.numpy()
    wq0, sw0 = orc.quantize_rows_sym(w)
    cs0 = orc.colsum_i8(wq0)
    mn0, mx0 = orc.range_f32(x)
    s0, z0 = orc.qparams_asym(mn0, mx0, 8)
    zx = z0 - 128
    xq0 = orc.quantize_act_i8(x, s0, zx)
    sr = float(np.float32(wl.w_std * np.linalg.norm(x[rows], axis=1).mean() / 30.0))
    zr = 3
    qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, float(s0), zx, sr, zr)
    m0 = torch.empty(n, dtype=torch.int32, device=DEV)
    sh = torch.empty(n, dtype=torch.int32, device=DEV)
    off = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_fold_fixed_point(dev(alpha), dev(beta), dev(sw0), dev(bias), dev(cs0), qp, m0, sh, off)
    m0_0, sh_0, off_0, _ = orc.fold_fixed_point(alpha, beta, sw0, bias, cs0, s0, zx, np.float32(sr))
    np.testing.assert_array_equal(host(m0), m0_0)
    np.testing.assert_array_equal(host(sh), sh_0)
    np.testing.assert_array_equal(host(off), off_0)
    out = torch.empty(m, n, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward_fixed_point(dev(xq0), dev(wq0), qp, m0, sh, off, out)
    acc = orc.gemm_i8(xq0[rows], wq0)
    want = orc.fixed_point_forward(acc, off_0, m0_0, sh_0, zr)
    got = host(out)
    np.testing.assert_array_equal(got[rows], want)
    # the fp32 epilogue of the same fold: at most one code apart, rarely
    mult, off_f, _ = orc.fold_int_offset(alpha, beta, sw0, bias, cs0, s0, zx, np.float32(sr))
    r_float = orc.folded_forward(acc, off_f, mult, zr).astype(np.int32)
    diff = np.abs(r_float - want.astype(np.int32))
    assert diff.max() <= 1 and np.mean(diff != 0) < 5e-3
