"""GPU parity: every entry point of the HIP library against the CPU oracle on the
same seeded inputs, through the C ABI.  Integer results (codes, accumulators,
offsets) must be bit-exact; fp32 statistics and (alpha, beta) within 1e-5
relative (scale-aware where the reference is near zero)."""

import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth
from cases import build_case
from tuning import tuning_of

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
RTOL = 1e-5  # tolerance stated by the benchmark spec for fp32 statistics and (alpha, beta)


def dev(a, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    P.binding.lib()  # fails loudly if the HIP library is missing


@pytest.fixture(scope="module")
def case1(orc):
    """Config 1 at its full size: 197 x 1152 x 384, 6304 calibration rows."""
    return build_case(orc, 1)


@pytest.fixture(scope="module")
def case5s(orc):
    """LLM-shaped (per-token scales, log-normal outlier channels), reduced."""
    return build_case(orc, 5, m=333, cal_rows=1536, n=1280, k=1024)


# --------------------------------------------------------------------------- quantizers
def test_range_and_quantize_act(orc, case1):
    c = case1
    x = dev(c.xcal)
    ws = torch.empty(P.cwac_range_workspace(x.numel()), dtype=torch.uint8, device=DEV)
    mm = torch.empty(2, dtype=torch.float32, device=DEV)
    P.cwac_range_f32(x, mm, ws)
    mn, mx = host(mm)
    assert (mn, mx) == orc.range_f32(c.xcal)
    s, z_u = P.cwac_qparams_from_range(float(mn), float(mx), 8)
    assert np.float32(s) == c.sx and z_u - 128 == c.zx
    for src, want in ((c.x, c.xq), (c.xcal, c.xq_cal)):
        q = torch.empty(src.shape, dtype=torch.int8, device=DEV)
        P.cwac_quantize_act(dev(src), s, z_u - 128, q)
        np.testing.assert_array_equal(host(q), want)


def test_quantize_act_ragged_layouts(orc):
    # odd width and padded leading dimensions take the element-wise path
    x = synth.normal(71, 0, 37 * 53).numpy().reshape(37, 53) * 3.0
    s, z = np.float32(0.05), -7
    want = orc.quantize_act_i8(x, s, z)
    xb = torch.zeros(37, 64, dtype=torch.float32, device=DEV)
    xb[:, :53] = dev(x)
    qb = torch.zeros(37, 60, dtype=torch.int8, device=DEV)
    P.cwac_quantize_act(xb[:, :53], float(s), z, qb[:, :53])
    np.testing.assert_array_equal(host(qb)[:, :53], want)
    assert np.all(host(qb)[:, 53:] == 0)               # padding untouched
    # a single-element tensor and its range
    one = dev(np.array([2.5], dtype=np.float32))
    mm = torch.empty(2, dtype=torch.float32, device=DEV)
    ws = torch.empty(P.cwac_range_workspace(1), dtype=torch.uint8, device=DEV)
    P.cwac_range_f32(one, mm, ws)
    assert tuple(host(mm)) == (2.5, 2.5)


def test_quantize_rows_sym_and_colsum(orc, case1, case5s):
    for c in (case1, case5s):
        w = dev(c.w)
        wq = torch.empty(c.w.shape, dtype=torch.int8, device=DEV)
        sw = torch.empty(c.n, dtype=torch.float32, device=DEV)
        P.cwac_quantize_rows_sym(w, sw, wq)
        np.testing.assert_array_equal(host(wq), c.wq)
        np.testing.assert_array_equal(host(sw), c.sw)
        cs = torch.empty(c.n, dtype=torch.int32, device=DEV)
        P.cwac_colsum(wq, cs)
        np.testing.assert_array_equal(host(cs), c.colsum)
    c = case5s                                          # per-token activations
    xq = torch.empty(c.x.shape, dtype=torch.int8, device=DEV)
    sx = torch.empty(c.m, dtype=torch.float32, device=DEV)
    P.cwac_quantize_rows_sym(dev(c.x), sx, xq)
    np.testing.assert_array_equal(host(xq), c.xq)
    np.testing.assert_array_equal(host(sx), c.sx_row)
    # odd width (element-wise path) and an all-zero row
    x = synth.normal(72, 0, 9 * 77).numpy().reshape(9, 77)
    x[4] = 0.0
    q0, s0 = orc.quantize_rows_sym(x)
    q = torch.empty(9, 77, dtype=torch.int8, device=DEV)
    s = torch.empty(9, dtype=torch.float32, device=DEV)
    P.cwac_quantize_rows_sym(dev(x), s, q)
    np.testing.assert_array_equal(host(q), q0)
    np.testing.assert_array_equal(host(s), s0)
    cs = torch.empty(9, dtype=torch.int32, device=DEV)
    P.cwac_colsum(q, cs)
    np.testing.assert_array_equal(host(cs), orc.colsum_i8(q0))


# --------------------------------------------------------------------------- forward
def _forward(c, out_kind, mult=None, offset=None, fbias=None, sx_row=None, qp=None, tile=None,
             xq=None, ldo=None, pipe=None, wgs=0, loaders=0):
    xq = c.xq if xq is None else xq
    m = xq.shape[0]
    dt = {0: torch.int8, 1: torch.float32, 2: torch.int32}[out_kind]
    if ldo is None:
        out = torch.empty(m, c.n, dtype=dt, device=DEV)
        view = out
    else:
        out = torch.full((m, ldo), 77, dtype=dt, device=DEV)
        view = out[:, :c.n]
    P.qlinear_cwac_forward(dev(xq), dev(c.wq), qp, dev(mult), dev(offset), dev(fbias),
                           dev(sx_row), out_kind, view, tuning=tuning_of(tile, pipe, persist_workgroups=wgs,
                                                                      persist_loaders=loaders))
    return host(out)


@pytest.mark.parametrize("tile", [64, 128, 256])
def test_forward_config1_all_modes(orc, case1, tile):
    c = case1
    acc = _forward(c, P.CWAC_OUT_INT32, tile=tile)
    np.testing.assert_array_equal(acc, c.acc)                        # raw accumulators
    acc_off = _forward(c, P.CWAC_OUT_INT32, offset=c.offset, tile=tile)
    np.testing.assert_array_equal(acc_off, c.acc + c.offset[None, :])
    qp = P.make_qparams(s_x=c.sx, z_x=c.zx, s_r=c.sr, z_r=c.zr)
    out = _forward(c, P.CWAC_OUT_INT8, c.mult, c.offset, qp=qp, tile=tile)
    np.testing.assert_array_equal(out, c.out)                        # folded CWAC, Eq. 10
    # plain PTQ parameters (alpha = 1, beta = 0) through the same kernel
    m0, o0, _ = orc.fold_int_offset(None, None, c.sw, c.bias, c.colsum, c.sx, c.zx, c.sr)
    out0 = _forward(c, P.CWAC_OUT_INT8, m0, o0, qp=qp, tile=tile)
    np.testing.assert_array_equal(out0, orc.folded_forward(c.acc, o0, m0, c.zr))
    # un-rounded beta
    mf, bf, of = orc.fold_fp_bias(c.alpha, c.beta, c.sw, c.bias, c.colsum, False, c.sx, c.zx, c.sr)
    out1 = _forward(c, P.CWAC_OUT_INT8, mf, of, fbias=bf, qp=qp, tile=tile)
    np.testing.assert_array_equal(out1, orc.folded_forward(c.acc, of, mf, c.zr, bf))
    # calibration forward: Y_quant in fp32, bit for bit
    md, bd, od = orc.fold_fp_bias(None, None, c.sw, c.bias, c.colsum, False, c.sx, c.zx, 1.0)
    yq = _forward(c, P.CWAC_OUT_FP32, md, od, fbias=bd, tile=tile, xq=c.xq_cal)
    np.testing.assert_array_equal(yq, c.y_quant)
    # narrow code range (4-bit codes in int8 containers)
    qp4 = P.make_qparams(s_x=c.sx, z_x=c.zx, s_r=c.sr, z_r=1, qmin=-8, qmax=7)
    out4 = _forward(c, P.CWAC_OUT_INT8, c.mult, c.offset, qp=qp4, tile=tile)
    np.testing.assert_array_equal(out4, orc.folded_forward(c.acc, c.offset, c.mult, 1,
                                                           qmin=-8, qmax=7))


@pytest.mark.parametrize("tile", [64, 128, 256])
def test_forward_per_token(orc, case5s, tile):
    c = case5s
    qp = P.make_qparams(mode=P.CWAC_EPI_FP_BIAS, act_per_token=True, s_r=c.sr, z_r=c.zr)
    out = _forward(c, P.CWAC_OUT_INT8, c.mult, c.offset, fbias=c.fbias, sx_row=c.sx_row, qp=qp,
                   tile=tile)
    np.testing.assert_array_equal(out, c.out)
    md, bd, od = orc.fold_fp_bias(None, None, c.sw, c.bias, c.colsum, True, 1.0, 0, 1.0)
    yq = _forward(c, P.CWAC_OUT_FP32, md, od, sx_row=c.sx_row_cal, tile=tile, xq=c.xq_cal)
    np.testing.assert_array_equal(yq, c.y_quant)


@pytest.mark.parametrize("m,n,k", [(1, 1, 16), (5, 3, 48), (70, 130, 144), (257, 259, 400),
                                   (300, 200, 96), (129, 513, 1040)])
def test_forward_ragged_shapes(orc, m, n, k):
    """Edges of every tile shape: odd M and N, K that is not a multiple of the K step,
    padded output rows (element-wise store path)."""
    g = synth.normal(900 + m, 0, m * k).numpy().reshape(m, k)
    xq = np.clip(np.rint(g * 60), -128, 127).astype(np.int8)
    g = synth.normal(900 + m, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 60), -127, 127).astype(np.int8)
    acc = orc.gemm_i8(xq, wq)
    mult = (np.abs(synth.normal(900 + m, 2, n).numpy()) * 1e-3 + 1e-4).astype(np.float32)
    off = np.rint(synth.normal(900 + m, 3, n).numpy() * 500).astype(np.int32)
    fb = synth.normal(900 + m, 4, n).numpy().astype(np.float32)
    sxr = (np.abs(synth.normal(900 + m, 5, m).numpy()) + 0.5).astype(np.float32)
    from types import SimpleNamespace
    c = SimpleNamespace(xq=xq, wq=wq, n=n)
    qp = P.make_qparams(z_r=-3)
    qpt = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, z_r=-3)      # per-row scales, fp bias
    for tile in (64, 128, 256):
        for ldo in (None, n + 3):
            got = _forward(c, P.CWAC_OUT_INT32, tile=tile, ldo=ldo)
            np.testing.assert_array_equal(got[:, :n], acc)
            if ldo:
                assert np.all(got[:, n:] == 77)          # nothing written past N
            got = _forward(c, P.CWAC_OUT_INT8, mult, off, qp=qp, tile=tile, ldo=ldo)
            np.testing.assert_array_equal(got[:, :n], orc.folded_forward(acc, off, mult, -3))
            got = _forward(c, P.CWAC_OUT_INT8, mult, off, fbias=fb, sx_row=sxr, qp=qpt, tile=tile,
                           ldo=ldo)
            np.testing.assert_array_equal(got[:, :n],
                                          orc.folded_forward(acc, off, mult, -3, fb, sxr))
            _, want = orc.folded_forward(acc, None, mult, 0, None, sxr, want_f32=True)
            got = _forward(c, P.CWAC_OUT_FP32, mult, sx_row=sxr, tile=tile, ldo=ldo)
            np.testing.assert_array_equal(got[:, :n], want)


@pytest.mark.parametrize("pipe", ["128x2", "64x4", "duo", "8w", "q", "persist"])
@pytest.mark.parametrize("m,n,k", [(256, 256, 128), (300, 520, 384), (700, 1030, 1152),
                                   (513, 768, 256),
                                   # K a multiple of 64 only: every pipe falls to the 64-byte K step
                                   (300, 520, 64), (520, 300, 192), (700, 256, 320),
                                   # fewer than 256 channels: the 256 x 128 tile, whatever the pipe
                                   (300, 128, 128), (520, 200, 192), (700, 255, 320),
                                   # fewer than 128: the 256 x 64 tile (64 x 64 wave tiles)
                                   (300, 64, 128), (520, 100, 192), (700, 127, 320)])
def test_forward_large_tile_kernel(orc, m, n, k, pipe):
    """The direct-to-LDS kernel (forced) in its three pipeline shapes - 256-token tiles with a
    128-byte or 64-byte K step, 128-token tiles with two workgroups per compute unit: edge tiles
    overlap their neighbours instead of being predicated; N not a multiple of 4 takes the
    element-wise stores."""
    print(f"large-tile kernel {pipe}: {m} x {n} x {k}", flush=True)
    g = synth.normal(700 + m, 0, m * k).numpy().reshape(m, k)
    xq = np.clip(np.rint(g * 60), -128, 127).astype(np.int8)
    g = synth.normal(700 + m, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 60), -127, 127).astype(np.int8)
    acc = orc.gemm_i8(xq, wq)
    mult = (np.abs(synth.normal(700 + m, 2, n).numpy()) * 1e-3 + 1e-4).astype(np.float32)
    off = np.rint(synth.normal(700 + m, 3, n).numpy() * 500).astype(np.int32)
    fb = synth.normal(700 + m, 4, n).numpy().astype(np.float32)
    sxr = (np.abs(synth.normal(700 + m, 5, m).numpy()) + 0.5).astype(np.float32)
    from types import SimpleNamespace
    c = SimpleNamespace(xq=xq, wq=wq, n=n)
    qp = P.make_qparams(z_r=5)
    qpt = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, z_r=5)
    for ldo in (None, n + 5):
        got = _forward(c, P.CWAC_OUT_INT32, tile="fast", ldo=ldo, pipe=pipe)
        np.testing.assert_array_equal(got[:, :n], acc)
        if ldo:
            assert np.all(got[:, n:] == 77)
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, qp=qp, tile="fast", ldo=ldo, pipe=pipe)
        np.testing.assert_array_equal(got[:, :n], orc.folded_forward(acc, off, mult, 5))
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, fbias=fb, sx_row=sxr, qp=qpt, tile="fast",
                       ldo=ldo, pipe=pipe)
        np.testing.assert_array_equal(got[:, :n], orc.folded_forward(acc, off, mult, 5, fb, sxr))
        _, want = orc.folded_forward(acc, off, mult, 0, fb, sxr, want_f32=True)
        got = _forward(c, P.CWAC_OUT_FP32, mult, off, fbias=fb, sx_row=sxr, tile="fast", ldo=ldo, pipe=pipe)
        np.testing.assert_array_equal(got[:, :n], want)


def test_forward_extreme_codes(orc):
    """All-extreme operands at the largest supported K: |acc| reaches K * 128 * 127."""
    m, n, k = 64, 96, 11008
    xq = np.full((m, k), -128, np.int8)
    wq = np.full((n, k), 127, np.int8)
    wq[1::2] = -127
    from types import SimpleNamespace
    c = SimpleNamespace(xq=xq, wq=wq, n=n)
    acc = _forward(c, P.CWAC_OUT_INT32)
    assert acc[0, 0] == -128 * 127 * k and acc[0, 1] == 128 * 127 * k
    np.testing.assert_array_equal(acc, orc.gemm_i8(xq, wq))


# --------------------------------------------------------------------------- statistics / fit
def _stats(yf, yq, splits=(None,)):
    n, c = yf.shape
    st = torch.empty(P.cwac_stats_bytes(c) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, c)
    bounds = [0] + [s for s in splits if s] + [n]
    for a, b in zip(bounds[:-1], bounds[1:]):
        ws = torch.empty(P.cwac_calibrate_stats_workspace(b - a, c), dtype=torch.uint8, device=DEV)
        P.cwac_calibrate_stats(yf[a:b], yq[a:b], st, ws)
    alpha = torch.empty(c, dtype=torch.float32, device=DEV)
    beta = torch.empty(c, dtype=torch.float32, device=DEV)
    mom = torch.empty(5, c, dtype=torch.float64, device=DEV)
    ndeg = torch.zeros(1, dtype=torch.int32, device=DEV)
    P.cwac_solve(st, c, alpha, beta, mom, ndeg)
    return host(alpha), host(beta), host(mom), int(host(ndeg)[0]), st


def _check_moments(mom, ref, rtol=RTOL):
    """Scale-aware relative error: means against the channel's spread, covariance
    against the product of spreads."""
    sf, sq = np.sqrt(ref[4]), np.sqrt(ref[2])
    floors = [sf, sq, sq * sq, sq * sf, sf * sf]
    for i in range(5):
        den = np.maximum(np.abs(ref[i]), floors[i]) + 1e-300
        err = np.abs(mom[i] - ref[i]) / den
        assert err.max() <= rtol, (i, err.max())


def _check_fit(alpha, beta, c, rtol=RTOL):
    sf = np.sqrt(c.moments[4])
    assert np.max(np.abs(alpha - c.alpha) / np.maximum(np.abs(c.alpha), 1.0)) <= rtol
    assert np.max(np.abs(beta - c.beta) / np.maximum(np.abs(c.beta), sf)) <= rtol


def test_stats_and_solve_config1(orc, case1):
    c = case1
    yf, yq = dev(c.y_full), dev(c.y_quant)
    alpha, beta, mom, ndeg, _ = _stats(yf, yq)
    _check_moments(mom, c.moments)
    _check_fit(alpha, beta, c)
    assert ndeg == c.n_degenerate == 0
    # streaming: three uneven batches give the same answer (fp64 summation order aside)
    a2, b2, mom2, _, _ = _stats(yf, yq, splits=(1000, 1001))
    _check_moments(mom2, c.moments)
    np.testing.assert_allclose(mom2, mom, rtol=1e-9, atol=1e-12)
    _check_fit(a2, b2, c)
    # degenerate channels spread over several workgroups of the solve kernel are all counted
    yq_c = c.y_quant.copy()
    yq_c[:, [3, 400, 1100]] = 0.5
    a4, _, _, nd4, _ = _stats(yf, dev(yq_c))
    assert nd4 == 3 and a4[3] == a4[400] == a4[1100] == 1.0
    # bit-reproducible for a given split
    a3, b3, mom3, _, _ = _stats(yf, yq)
    np.testing.assert_array_equal(mom3, mom)
    np.testing.assert_array_equal(a3, alpha)


def test_stats_per_token_case(orc, case5s):
    c = case5s
    alpha, beta, mom, ndeg, _ = _stats(dev(c.y_full), dev(c.y_quant))
    _check_moments(mom, c.moments)
    _check_fit(alpha, beta, c)


def test_stats_generic_layout_and_hard_channels(orc):
    """Odd channel count with padded rows (generic kernel); channels whose mean is
    1e5 times their spread; constant channels (degenerate fallback)."""
    rows, ch = 1537, 30
    yq = synth.normal(81, 0, rows * ch).numpy().reshape(rows, ch).astype(np.float32)
    e = synth.normal(81, 1, rows * ch).numpy().reshape(rows, ch)
    yq[:, 3] = yq[:, 3] * 0.01 + 1000.0
    yf = (1.1 * yq + 0.2 + 0.05 * e).astype(np.float32)
    yf[:, 3] = (yq[:, 3].astype(np.float64) + 0.002 * e[:, 3]).astype(np.float32)
    yq[:, 7] = 2.0
    yf[:, 9] = -1.0
    ref = orc.channel_moments(yf, yq)
    a0, b0, nd0 = orc.solve(ref)
    fb = torch.zeros(rows, 37, dtype=torch.float32, device=DEV)
    qb = torch.zeros(rows, 33, dtype=torch.float32, device=DEV)
    fb[:, :ch] = dev(yf)
    qb[:, :ch] = dev(yq)
    alpha, beta, mom, ndeg, _ = _stats(fb[:, :ch], qb[:, :ch], splits=(700,))
    _check_moments(mom, ref)
    assert ndeg == nd0 == 2
    sf = np.sqrt(ref[4])
    assert np.max(np.abs(alpha - a0) / np.maximum(np.abs(a0), 1.0)) <= RTOL
    assert np.max(np.abs(beta - b0) / np.maximum(np.abs(b0), np.maximum(sf, 1e-30))) <= RTOL
    assert alpha[7] == 1.0 and alpha[9] == 1.0
    # the same data through the vector kernel (channels padded to a multiple of 4)
    f4 = torch.zeros(rows, 32, dtype=torch.float32, device=DEV)
    q4 = torch.zeros(rows, 32, dtype=torch.float32, device=DEV)
    f4[:, :ch] = dev(yf)
    q4[:, :ch] = dev(yq)
    _, _, mom4, _, _ = _stats(f4, q4)
    _check_moments(mom4[:, :ch], ref)


@pytest.mark.parametrize("rows,ch", [(60000, 64), (20000, 1024), (3000, 4096), (2500, 200), (40000, 1000)])
def test_stats_merge_every_width(orc, rows, ch):
    """Row-group counts on either side of the merge kernel's widths (235, 78, 12, 10 and 157 partial sums per
    channel) and channel counts that leave tasks of the last merge workgroup empty."""
    print(f"statistics {rows} x {ch}", flush=True)
    yq = synth.normal(83 + ch, 0, rows * ch).numpy().reshape(rows, ch).astype(np.float32)
    e = synth.normal(83 + ch, 1, rows * ch).numpy().reshape(rows, ch)
    yf = (0.9 * yq - 0.1 + 0.1 * e).astype(np.float32)
    ref = orc.channel_moments(yf, yq)
    a0, b0, _ = orc.solve(ref)
    alpha, beta, mom, ndeg, _ = _stats(dev(yf), dev(yq), splits=(rows // 3,))
    _check_moments(mom, ref)
    assert ndeg == 0
    sf = np.sqrt(ref[4])
    assert np.max(np.abs(alpha - a0) / np.maximum(np.abs(a0), 1.0)) <= RTOL
    assert np.max(np.abs(beta - b0) / np.maximum(np.abs(b0), sf)) <= RTOL


def test_stats_empty_state_and_single_row(orc):
    ch = 8
    st = torch.empty(P.cwac_stats_bytes(ch) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, ch)
    alpha = torch.empty(ch, dtype=torch.float32, device=DEV)
    beta = torch.empty(ch, dtype=torch.float32, device=DEV)
    ndeg = torch.zeros(1, dtype=torch.int32, device=DEV)
    P.cwac_solve(st, ch, alpha, beta, None, ndeg)          # no rows: identity, all degenerate
    assert np.all(host(alpha) == 1.0) and np.all(host(beta) == 0.0) and int(host(ndeg)[0]) == ch
    yf = dev(np.arange(8, dtype=np.float32)[None, :])
    yq = dev(np.arange(8, dtype=np.float32)[None, :] * 0.5)
    a, b, mom, nd, _ = _stats(yf, yq)                       # one row: variance 0 -> shift only
    assert np.all(a == 1.0) and nd == ch
    np.testing.assert_array_equal(b, np.arange(8, dtype=np.float32) * 0.5)


@pytest.mark.parametrize("wgs", [1, 3, 5, 7, 11, 0])
@pytest.mark.parametrize("m,n,k", [(1300, 1030, 512), (600, 780, 128), (777, 520, 256), (520, 1290, 384),
                                   (1030, 600, 1152), (520, 780, 4096), (777, 520, 4224)])
def test_forward_persistent_tiles(orc, m, n, k, wgs):
    """The persistent form of the 256 x 256 tile with fewer workgroups than tiles, so that every
    workgroup walks several tiles (the next tile's first loads in flight under a tile's epilogue):
    one to nine K stages (odd and even: the last stage ends in either ring buffer), ragged edge
    tiles, every output kind, padded output rows; from K = 4096 the form in which four of the eight
    wavefronts issue all panel loads (32 and 33 stages)."""
    print(f"persistent tiles {m} x {n} x {k}, {wgs or 'one per CU'} workgroups", flush=True)
    g = synth.normal(1700 + m, 0, m * k).numpy().reshape(m, k)
    xq = np.clip(np.rint(g * 60), -128, 127).astype(np.int8)
    g = synth.normal(1700 + m, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 60), -127, 127).astype(np.int8)
    acc = orc.gemm_i8(xq, wq)
    mult = (np.abs(synth.normal(1700 + m, 2, n).numpy()) * 1e-3 + 1e-4).astype(np.float32)
    off = np.rint(synth.normal(1700 + m, 3, n).numpy() * 500).astype(np.int32)
    fb = synth.normal(1700 + m, 4, n).numpy().astype(np.float32)
    sxr = (np.abs(synth.normal(1700 + m, 5, m).numpy()) + 0.5).astype(np.float32)
    from types import SimpleNamespace
    c = SimpleNamespace(xq=xq, wq=wq, n=n)
    zr = -6 if wgs in (0, 3) else 5      # even and odd: the zero point reaches the code in two different ways
    qp = P.make_qparams(z_r=zr)
    qpt = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, z_r=zr)
    kw = dict(tile="fast", pipe="persist", wgs=wgs)
    for ldo in (None, n + 5):
        got = _forward(c, P.CWAC_OUT_INT32, offset=off, ldo=ldo, **kw)
        np.testing.assert_array_equal(got[:, :n], acc + off[None, :])
        if ldo:
            assert np.all(got[:, n:] == 77)
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, qp=qp, ldo=ldo, **kw)
        np.testing.assert_array_equal(got[:, :n], orc.folded_forward(acc, off, mult, zr))
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, fbias=fb, sx_row=sxr, qp=qpt, ldo=ldo, **kw)
        np.testing.assert_array_equal(got[:, :n], orc.folded_forward(acc, off, mult, zr, fb, sxr))
        _, want = orc.folded_forward(acc, off, mult, 0, fb, sxr, want_f32=True)
        got = _forward(c, P.CWAC_OUT_FP32, mult, off, fbias=fb, sx_row=sxr, ldo=ldo, **kw)
        np.testing.assert_array_equal(got[:, :n], want)
    # the count of loading wavefronts that the launcher would not pick at this K, forced through cwac_tuning
    other = 8 if k >= 4096 else 4
    got = _forward(c, P.CWAC_OUT_INT8, mult, off, qp=qp, loaders=other, **kw)
    np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, zr))
    got = _forward(c, P.CWAC_OUT_INT8, mult, off, fbias=fb, sx_row=sxr, qp=qpt, loaders=other, **kw)
    np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, zr, fb, sxr))
    got = _forward(c, P.CWAC_OUT_INT32, offset=off, loaders=other, **kw)
    np.testing.assert_array_equal(got, acc + off[None, :])


@pytest.mark.parametrize("m,n,k,wgs", [(25216, 768, 256, 0), (4500, 1100, 384, 64), (2100, 512, 128, 16),
                                       (2100, 512, 4224, 16)])
def test_forward_persistent_last_round_in_quarters(orc, m, n, k, wgs):
    """A last round of at most a quarter of the workgroups: its tiles are cut into four items of 64 tokens (short
    K loops; with K >= 4096 into two halves unless eight loading wavefronts are forced).  Full grid of one
    workgroup per compute unit (297 tiles, 41 of them in the last round) and smaller grids; ragged edges;
    per-tensor and per-token epilogues, int8 and fp32 out."""
    print(f"persistent tiles, quartered last round {m} x {n} x {k}, {wgs or 'one per CU'} workgroups", flush=True)
    g = synth.normal(1900 + k, 0, m * k).numpy().reshape(m, k)
    xq = np.clip(np.rint(g * 40), -128, 127).astype(np.int8)
    g = synth.normal(1900 + k, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 40), -127, 127).astype(np.int8)
    acc = orc.gemm_i8(xq, wq)
    mult = (np.abs(synth.normal(1900 + k, 2, n).numpy()) * 1e-3 + 1e-4).astype(np.float32)
    off = np.rint(synth.normal(1900 + k, 3, n).numpy() * 500).astype(np.int32)
    fb = synth.normal(1900 + k, 4, n).numpy().astype(np.float32)
    sxr = (np.abs(synth.normal(1900 + k, 5, m).numpy()) + 0.5).astype(np.float32)
    from types import SimpleNamespace
    c = SimpleNamespace(xq=xq, wq=wq, n=n)
    qp = P.make_qparams(z_r=-3)
    qpt = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, z_r=-3)
    for loaders in (0, 8):
        kw = dict(tile="fast", pipe="persist", wgs=wgs, loaders=loaders)
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, qp=qp, **kw)
        np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, -3))
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, fbias=fb, sx_row=sxr, qp=qpt, ldo=n + 16, **kw)
        np.testing.assert_array_equal(got[:, :n], orc.folded_forward(acc, off, mult, -3, fb, sxr))
        assert np.all(got[:, n:] == 77)
        _, want = orc.folded_forward(acc, off, mult, 0, fb, sxr, want_f32=True)
        got = _forward(c, P.CWAC_OUT_FP32, mult, off, fbias=fb, sx_row=sxr, **kw)
        np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("zr", [-128, -77, -6, 0, 1, 5, 126, 127])
def test_forward_ties_and_saturation_for_every_zero_point_parity(orc, zr):
    """Multipliers that are powers of two and biases that are multiples of 1/2 put many results exactly half
    way between two codes (round half to even decides), and a few channels saturate at either end; even and
    odd zero points, at the ends of their range too.  Persistent tile and the one-workgroup-per-tile form."""
    m, n, k = 520, 512, 256
    print(f"ties and saturation, z_r = {zr}", flush=True)
    g = synth.normal(2100, 0, m * k).numpy().reshape(m, k)
    xq = np.clip(np.rint(g * 3), -128, 127).astype(np.int8)
    g = synth.normal(2100, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 3), -127, 127).astype(np.int8)
    acc = orc.gemm_i8(xq, wq)
    mult = np.array([0.5, 0.25, 0.125, -0.5, 1.5, 0.0625, 4.0, -8.0], dtype=np.float32)[np.arange(n) % 8]
    off = np.rint(synth.normal(2100, 3, n).numpy() * 50).astype(np.int32)
    fb = (np.rint(synth.normal(2100, 4, n).numpy() * 20) * 0.5).astype(np.float32)
    sxr = np.array([1.0, 0.5, 2.0, 0.25], dtype=np.float32)[np.arange(m) % 4]
    want = orc.folded_forward(acc, off, mult, zr)
    u = (acc + off[None, :]).astype(np.float64) * mult[None, :].astype(np.float64)
    assert np.mean(np.abs(u - np.floor(u)) == 0.5) > 0.1          # the case does hold exact ties
    assert (want == -128).any() and (want == 127).any()           # and both ends
    from types import SimpleNamespace
    c = SimpleNamespace(xq=xq, wq=wq, n=n)
    qp = P.make_qparams(z_r=zr)
    qpt = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, z_r=zr)
    for pipe in ("persist", "8w"):
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, qp=qp, tile="fast", pipe=pipe)
        np.testing.assert_array_equal(got, want)
        got = _forward(c, P.CWAC_OUT_INT8, mult, off, fbias=fb, sx_row=sxr, qp=qpt, tile="fast", pipe=pipe)
        np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, zr, fb, sxr))


# --------------------------------------------------------------------------- fold
def test_fold_bit_exact(orc, case1, case5s):
    for c in (case1, case5s):
        n = c.n
        mult = torch.empty(n, dtype=torch.float32, device=DEV)
        off = torch.empty(n, dtype=torch.int32, device=DEV)
        fb = torch.empty(n, dtype=torch.float32, device=DEV)
        nsat = torch.zeros(1, dtype=torch.int32, device=DEV)
        args = (dev(c.sw), dev(c.bias), dev(c.colsum))
        if not c.per_token:
            qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, c.sx, c.zx, c.sr, c.zr)
            alpha = c.alpha.copy()
            alpha[5] = 1e-30                                   # forces a saturated offset
            P.cwac_fold(dev(alpha), dev(c.beta), *args, qp, mult, off, None, nsat)
            m0, o0, ns0 = orc.fold_int_offset(alpha, c.beta, c.sw, c.bias, c.colsum, c.sx, c.zx, c.sr)
            np.testing.assert_array_equal(host(mult), m0)
            np.testing.assert_array_equal(host(off), o0)
            assert int(host(nsat)[0]) == ns0 == 1
            P.cwac_fold(None, None, *args, qp, mult, off, None, None)   # plain PTQ (Eq. 7-8)
            m0, o0, _ = orc.fold_int_offset(None, None, c.sw, c.bias, c.colsum, c.sx, c.zx, c.sr)
            np.testing.assert_array_equal(host(mult), m0)
            np.testing.assert_array_equal(host(off), o0)
        qp = P.make_qparams(P.CWAC_EPI_FP_BIAS, c.per_token, c.sx, c.zx, c.sr, c.zr)
        P.cwac_fold(dev(c.alpha), dev(c.beta), *args, qp, mult, off, fb, None)
        m1, b1, o1 = orc.fold_fp_bias(c.alpha, c.beta, c.sw, c.bias, c.colsum, c.per_token,
                                      c.sx, c.zx, c.sr)
        np.testing.assert_array_equal(host(mult), m1)
        np.testing.assert_array_equal(host(fb), b1)
        np.testing.assert_array_equal(host(off), o1)
        qp = P.make_qparams(P.CWAC_EPI_FP_BIAS, c.per_token, c.sx, c.zx, 1.0, 0)
        P.cwac_fold(None, None, *args, qp, mult, off, fb, None)         # dequantization parameters
        np.testing.assert_array_equal(host(mult), c.deq)


# --------------------------------------------------------------------------- un-fused comparators
def test_unfused_epilogue_and_affine(orc, case1, case5s):
    c = case1
    qp = P.make_qparams(s_x=c.sx, z_x=c.zx, s_r=c.sr, z_r=c.zr)
    out = torch.empty(c.m, c.n, dtype=torch.int8, device=DEV)
    P.cwac_epilogue_int32(dev(c.acc), qp, dev(c.mult), dev(c.offset), None, None, P.CWAC_OUT_INT8, out)
    np.testing.assert_array_equal(host(out), c.out)
    c = case5s
    qp = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, s_r=c.sr, z_r=c.zr)
    out = torch.empty(c.m, c.n, dtype=torch.int8, device=DEV)
    P.cwac_epilogue_int32(dev(c.acc), qp, dev(c.mult), dev(c.offset), dev(c.fbias), dev(c.sx_row),
                          P.CWAC_OUT_INT8, out)
    np.testing.assert_array_equal(host(out), c.out)
    pad = torch.zeros(c.m, c.n + 1, dtype=torch.float32, device=DEV)    # element-wise path
    P.cwac_epilogue_int32(dev(c.acc), None, dev(c.mult), dev(c.offset), dev(c.fbias),
                          dev(c.sx_row), P.CWAC_OUT_FP32, pad[:, :c.n])
    _, u = orc.folded_forward(c.acc, c.offset, c.mult, 0, c.fbias, c.sx_row, want_f32=True)
    np.testing.assert_array_equal(host(pad)[:, :c.n], u)
    yc = torch.empty(c.cal_rows, c.n, dtype=torch.float32, device=DEV)
    P.cwac_apply_unfolded(dev(c.y_quant), dev(c.alpha), dev(c.beta), yc)
    np.testing.assert_array_equal(host(yc), orc.cwac_apply(c.y_quant, c.alpha, c.beta))


# --------------------------------------------------------------------------- whole pipeline on the device
def _device_pipeline(c, wl_per_token):
    """quantize -> calibration forward -> statistics -> fit -> fold -> folded forward,
    every step in the HIP library, from the same fp32 tensors the oracle case used."""
    n, k = c.n, c.k
    wq = torch.empty(n, k, dtype=torch.int8, device=DEV)
    sw = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_quantize_rows_sym(dev(c.w), sw, wq)
    colsum = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_colsum(wq, colsum)
    bias = dev(c.bias)
    xq = torch.empty(c.m, k, dtype=torch.int8, device=DEV)
    xq_cal = torch.empty(c.cal_rows, k, dtype=torch.int8, device=DEV)
    if wl_per_token:
        sx_row = torch.empty(c.m, dtype=torch.float32, device=DEV)
        sx_row_cal = torch.empty(c.cal_rows, dtype=torch.float32, device=DEV)
        P.cwac_quantize_rows_sym(dev(c.x), sx_row, xq)
        P.cwac_quantize_rows_sym(dev(c.xcal), sx_row_cal, xq_cal)
        sx, zx = 1.0, 0
    else:
        xcal = dev(c.xcal)
        mm = torch.empty(2, dtype=torch.float32, device=DEV)
        ws = torch.empty(P.cwac_range_workspace(xcal.numel()), dtype=torch.uint8, device=DEV)
        P.cwac_range_f32(xcal, mm, ws)
        mn, mx = host(mm)
        sx, z_u = P.cwac_qparams_from_range(float(mn), float(mx), 8)
        zx = z_u - 128
        P.cwac_quantize_act(dev(c.x), sx, zx, xq)
        P.cwac_quantize_act(xcal, sx, zx, xq_cal)
        sx_row = sx_row_cal = None
    mult = torch.empty(n, dtype=torch.float32, device=DEV)
    off = torch.empty(n, dtype=torch.int32, device=DEV)
    fb = torch.empty(n, dtype=torch.float32, device=DEV)
    qp_deq = P.make_qparams(P.CWAC_EPI_FP_BIAS, wl_per_token, sx, zx, 1.0, 0)
    P.cwac_fold(None, None, sw, bias, colsum, qp_deq, mult, off, fb, None)
    yq = torch.empty(c.cal_rows, n, dtype=torch.float32, device=DEV)
    P.qlinear_cwac_forward(xq_cal, wq, None, mult, off, fb if bias is not None else None,
                           sx_row_cal, P.CWAC_OUT_FP32, yq)
    st = torch.empty(P.cwac_stats_bytes(n) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, n)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(c.cal_rows, n), dtype=torch.uint8, device=DEV)
    P.cwac_calibrate_stats(dev(c.y_full), yq, st, ws)
    alpha = torch.empty(n, dtype=torch.float32, device=DEV)
    beta = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_solve(st, n, alpha, beta)
    return dict(wq=wq, sw=sw, colsum=colsum, bias=bias, xq=xq, sx_row=sx_row, sx=sx, zx=zx,
                yq=yq, alpha=alpha, beta=beta)


def test_pipeline_on_device_config1(orc, case1):
    c = case1
    d = _device_pipeline(c, False)
    np.testing.assert_array_equal(host(d["yq"]), c.y_quant)
    _check_fit(host(d["alpha"]), host(d["beta"]), c)
    # fold the DEVICE-side (alpha, beta); the oracle folds the same values -> identical codes
    a, b = host(d["alpha"]), host(d["beta"])
    qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, d["sx"], d["zx"], c.sr, c.zr)
    mult = torch.empty(c.n, dtype=torch.float32, device=DEV)
    off = torch.empty(c.n, dtype=torch.int32, device=DEV)
    P.cwac_fold(d["alpha"], d["beta"], d["sw"], d["bias"], d["colsum"], qp, mult, off)
    out = torch.empty(c.m, c.n, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward(d["xq"], d["wq"], qp, mult, off, None, None, P.CWAC_OUT_INT8, out)
    m0, o0, _ = orc.fold_int_offset(a, b, c.sw, c.bias, c.colsum, c.sx, c.zx, c.sr)
    np.testing.assert_array_equal(host(out), orc.folded_forward(c.acc, o0, m0, c.zr))
    # and against the oracle's own end-to-end codes: (alpha, beta) differ by <= 1e-5 relative,
    # which moves a code only next to a rounding boundary
    diff = host(out).astype(np.int32) - c.out.astype(np.int32)
    assert np.max(np.abs(diff)) <= 1 and np.mean(diff != 0) < 1e-3


def test_pipeline_on_device_per_token(orc, case5s):
    c = case5s
    d = _device_pipeline(c, True)
    np.testing.assert_array_equal(host(d["yq"]), c.y_quant)
    _check_fit(host(d["alpha"]), host(d["beta"]), c)
    a, b = host(d["alpha"]), host(d["beta"])
    qp = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, 1.0, 0, c.sr, c.zr)
    mult = torch.empty(c.n, dtype=torch.float32, device=DEV)
    off = torch.empty(c.n, dtype=torch.int32, device=DEV)
    fb = torch.empty(c.n, dtype=torch.float32, device=DEV)
    P.cwac_fold(d["alpha"], d["beta"], d["sw"], None, d["colsum"], qp, mult, off, fb)
    out = torch.empty(c.m, c.n, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward(d["xq"], d["wq"], qp, mult, off, fb, d["sx_row"], P.CWAC_OUT_INT8, out)
    m1, b1, o1 = orc.fold_fp_bias(a, b, c.sw, None, c.colsum, True, 1.0, 0, c.sr)
    np.testing.assert_array_equal(host(out), orc.folded_forward(c.acc, o1, m1, c.zr, b1, c.sx_row))
