"""GPU parity of the weight-only INT4 layer (LLM setting of Sec. 4.4 with the CWAC of
Sec. 3.3-3.4) against the CPU oracle, through the C ABI.

Integer work (codes, zero-points, scale bit patterns, fold constants) is compared bit for
bit.  The layer product is accumulated in fp32 on the matrix cores in an unspecified order,
so it is checked two ways: on operands whose every partial sum is exactly representable
(then any summation order gives the same bits, and outputs must EQUAL the oracle's), and on
workload-like operands against the exact fp64 product within
    8 * sqrt(K) * 2^-24 * sum_k |x w|        (fp32 summation, probabilistic bound with margin)
plus the roundings of the two epilogue operations and of the binary16 store."""
import os

import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth
from tuning import tuning_of, w4_pipes

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
U = 2.0 ** -24


@pytest.fixture(scope="module")
def w4():
    from oracle import w4a16_oracle
    w4a16_oracle.build()
    return w4a16_oracle


def _dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _pack(codes, scales, zeros):
    n, k = codes.shape
    pw = torch.empty(P.cwac_w4_packed_w_bytes(n, k), dtype=torch.uint8, device=DEV)
    psz = torch.empty((k // 128) * n, dtype=torch.int32, device=DEV)
    P.cwac_w4_pack(_dev(codes), _dev(scales), _dev(zeros), pw, psz)
    return pw, psz


def _forward(x16, pw, psz, n, mult, fbias, dtype, ldo=None, pipe=None, waves=0, depth=0):
    m = x16.shape[0]
    if ldo is None:
        out = torch.empty(m, n, dtype=dtype, device=DEV)
    else:
        full = torch.full((m, ldo), 7.0, dtype=dtype, device=DEV)
        out = full[:, :n]
    P.qlinear_w4a16_cwac_forward(_dev(x16), pw, psz, n, _dev(mult), _dev(fbias), out,
                                 tuning=tuning_of(w4_pipe=pipe, w4_small_waves=waves, w4_small_depth=depth))
    torch.cuda.synchronize()
    if ldo is not None:
        assert (full[:, n:] == 7.0).all(), "wrote outside the output columns"
    return out


# ------------------------------------------------------------------ quantizer, packing, fold
def test_group_quantizer_bit_exact(w4):
    n, k = 96, 1024
    w = (synth.normal(41, 1, n * k).numpy() * 0.02).reshape(n, k).copy()
    w[3, 128:256] += 0.07          # zero-point clips at 0
    w[4, 0:128] -= 0.09            # zero-point clips at 15
    w[5, 256:384] = 0.125          # constant group: scale floored at 2^-14
    w[6, 384:512] *= 1e-7          # scale below the binary16 normal range
    w[7, 512:640] *= 3e6           # scale beyond the binary16 range
    codes0, scales0, zeros0 = w4.quantize_groupwise(w)
    codes = torch.empty(n, k, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n, k // 128, dtype=torch.float16, device=DEV)
    zeros = torch.empty(n, k // 128, dtype=torch.uint8, device=DEV)
    P.cwac_w4_quantize_groupwise(_dev(w), codes, scales, zeros)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(scales.cpu().numpy().view(np.uint16), scales0.view(np.uint16))
    np.testing.assert_array_equal(zeros.cpu().numpy(), zeros0)
    np.testing.assert_array_equal(codes.cpu().numpy(), codes0)
    # padded leading dimension
    wp = torch.zeros(n, k + 64, dtype=torch.float32, device=DEV)
    wp[:, :k] = _dev(w)
    codes.zero_()
    P.cwac_w4_quantize_groupwise(wp[:, :k], codes, scales, zeros)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(codes.cpu().numpy(), codes0)


def test_packed_layout_is_the_documented_one():
    """cwac.h states the streaming layout; unpack it here from that description."""
    rng = np.random.default_rng(2)
    n, k = 64, 256
    codes = rng.integers(0, 16, (n, k), dtype=np.uint8)
    scales = (rng.random((n, k // 128)) + 0.5).astype(np.float16)
    zeros = rng.integers(0, 16, (n, k // 128), dtype=np.uint8)
    pw, psz = _pack(codes, scales, zeros)
    words = pw.cpu().numpy().view(np.uint32).reshape(n // 32, k // 64, 64, 4)
    nib = (0, 4, 1, 5, 2, 6, 3, 7)
    got = np.zeros_like(codes)
    for nb in range(n // 32):
        for kb in range(k // 64):
            for lane in range(64):
                h, r = lane // 32, lane % 32
                for j in range(4):
                    wd = int(words[nb, kb, lane, j])
                    for e in range(8):
                        got[nb * 32 + r, kb * 64 + 16 * j + 8 * h + e] = (wd >> (4 * nib[e])) & 15
    np.testing.assert_array_equal(got, codes)
    sz = psz.cpu().numpy().view(np.uint32).reshape(k // 128, n)
    np.testing.assert_array_equal((sz & 0xffff).astype(np.uint16).T, scales.view(np.uint16))
    np.testing.assert_array_equal((sz >> 16).astype(np.uint8).T, zeros)


def test_fold_weight_only_bit_exact(w4):
    n = 700
    alpha = (1 + 0.1 * synth.normal(42, 0, n).numpy()).astype(np.float32)
    beta = (0.05 * synth.normal(42, 1, n).numpy()).astype(np.float32)
    bias = (0.02 * synth.normal(42, 2, n).numpy()).astype(np.float32)
    mult = torch.empty(n, dtype=torch.float32, device=DEV)
    fbias = torch.empty(n, dtype=torch.float32, device=DEV)
    for a, be, b in [(alpha, beta, bias), (alpha, beta, None), (None, None, bias), (None, None, None)]:
        P.cwac_fold_weight_only(_dev(a), _dev(be), _dev(b), mult, fbias)
        torch.cuda.synchronize()
        m0, f0 = w4.fold(a, be, b, n)
        np.testing.assert_array_equal(mult.cpu().numpy(), m0)
        np.testing.assert_array_equal(fbias.cpu().numpy(), f0)
    with pytest.raises(P.CwacError):
        P.cwac_fold_weight_only(_dev(alpha), None, None, mult, fbias)


# ------------------------------------------------------------------ forward: exact operands
def _exact_case(seed, m, n, k):
    """Small-integer activations, power-of-two scales: every product and every partial sum is
    exactly representable in fp32, whatever the order of summation."""
    rng = np.random.default_rng(seed)
    x16 = rng.integers(-3, 4, (m, k)).astype(np.float16)
    codes = rng.integers(0, 16, (n, k), dtype=np.uint8)
    zeros = rng.integers(0, 16, (n, k // 128), dtype=np.uint8)
    scales = (2.0 ** rng.integers(-3, 4, (n, k // 128))).astype(np.float16)
    return x16, codes, scales, zeros


@pytest.mark.parametrize("m,n,k", [(256, 256, 128), (300, 512, 384), (1, 256, 256), (513, 288, 256),
                                   (77, 800, 1024), (1024, 256, 2048), (129, 544, 640), (385, 256, 512),
                                   (700, 1056, 256), (128, 512, 128), (260, 1024, 1152)])
def test_forward_exact_operands(w4, m, n, k):
    print(f"w4a16 exact operands {m} x {n} x {k}", flush=True)
    x16, codes, scales, zeros = _exact_case(100 + m + n + k, m, n, k)
    wd = w4.dequant(codes, scales, zeros)
    acc, _ = w4.product(x16, wd)
    acc32 = acc.astype(np.float32)
    assert np.array_equal(acc32.astype(np.float64), acc)          # exactly representable
    pw, psz = _pack(codes, scales, zeros)
    rng = np.random.default_rng(5)
    mult = (1 + 0.25 * rng.standard_normal(n)).astype(np.float32)
    fbias = rng.standard_normal(n).astype(np.float32)
    o32, o16 = w4.epilogue_f32(acc32, mult, fbias)
    o32m, _ = w4.epilogue_f32(acc32, mult, None)
    o32b, _ = w4.epilogue_f32(acc32, None, fbias)
    # the automatic choice, then the 256-token and the 128-token tile forced
    for pipe in w4_pipes(n):
        # raw product, fp32 out
        out = _forward(x16, pw, psz, n, None, None, torch.float32, pipe=pipe)
        np.testing.assert_array_equal(out.cpu().numpy(), acc32)
        # folded epilogue, fp32 and binary16 out, padded output pitch
        out = _forward(x16, pw, psz, n, mult, fbias, torch.float32, ldo=n + 12, pipe=pipe)
        np.testing.assert_array_equal(out.cpu().numpy(), o32)
        outh = _forward(x16, pw, psz, n, mult, fbias, torch.float16, ldo=n + 24, pipe=pipe)
        np.testing.assert_array_equal(outh.cpu().numpy().view(np.uint16), o16.view(np.uint16))
        # only one of the two epilogue vectors
        np.testing.assert_array_equal(
            _forward(x16, pw, psz, n, mult, None, torch.float32, pipe=pipe).cpu().numpy(), o32m)
        np.testing.assert_array_equal(
            _forward(x16, pw, psz, n, None, fbias, torch.float32, pipe=pipe).cpu().numpy(), o32b)


@pytest.mark.parametrize("n,k", [(256, 128), (320, 384), (512, 1024), (288, 640)])
@pytest.mark.parametrize("m", [1, 5, 17, 32])
def test_small_batch_exact_operands(w4, m, n, k):
    """Batches of at most 32 tokens take the weight-streaming kernel (one workgroup per 32 channels,
    K split over its four wavefronts - here 1, 3, 8 and 5 groups); `tile` and `half` force the tiled kernel
    with 256- and 128-token tiles.
    Exact operands: both give the oracle's bits."""
    print(f"w4a16 small batch {m} x {n} x {k}", flush=True)
    x16, codes, scales, zeros = _exact_case(300 + m + n + k, m, n, k)
    wd = w4.dequant(codes, scales, zeros)
    acc, _ = w4.product(x16, wd)
    acc32 = acc.astype(np.float32)
    assert np.array_equal(acc32.astype(np.float64), acc)
    pw, psz = _pack(codes, scales, zeros)
    rng = np.random.default_rng(6)
    mult = (1 + 0.25 * rng.standard_normal(n)).astype(np.float32)
    fbias = rng.standard_normal(n).astype(np.float32)
    o32, o16 = w4.epilogue_f32(acc32, mult, fbias)
    o32m, _ = w4.epilogue_f32(acc32, mult, None)
    o32b, _ = w4.epilogue_f32(acc32, None, fbias)
    for pipe in w4_pipes(n):
        out = _forward(x16, pw, psz, n, None, None, torch.float32, pipe=pipe)
        np.testing.assert_array_equal(out.cpu().numpy(), acc32)
        out = _forward(x16, pw, psz, n, mult, fbias, torch.float32, ldo=n + 12, pipe=pipe)
        np.testing.assert_array_equal(out.cpu().numpy(), o32)
        outh = _forward(x16, pw, psz, n, mult, fbias, torch.float16, ldo=n + 24, pipe=pipe)
        np.testing.assert_array_equal(outh.cpu().numpy().view(np.uint16), o16.view(np.uint16))
        np.testing.assert_array_equal(
            _forward(x16, pw, psz, n, mult, None, torch.float32, pipe=pipe).cpu().numpy(), o32m)
        np.testing.assert_array_equal(
            _forward(x16, pw, psz, n, None, fbias, torch.float32, pipe=pipe).cpu().numpy(), o32b)


@pytest.mark.parametrize("waves,depth", [(4, 0), (8, 0), (4, 2), (8, 2), (4, 3), (8, 3), (4, 4), (8, 4)])
@pytest.mark.parametrize("m,n,k", [(1, 256, 128), (7, 288, 640), (32, 256, 1152), (19, 320, 2560), (32, 256, 4224),
                                   (3, 256, 9088), (8, 256, 2048), (9, 256, 1536), (16, 288, 3072), (13, 256, 4224)])
def test_small_batch_every_wave_count(w4, m, n, k, waves, depth):
    """The weight-streaming kernel with 4 and 8 wavefronts per workgroup and every ring depth, for each padded row
    count (8, 16, 32; by default rings of 4, 3 and 3 groups per wavefront): wavefronts without a group (K = 128), with fewer groups than ring
    slots, with exactly a ring, and with several rounds of the ring plus a ragged rest (33 and 71 groups).  Exact
    operands: the oracle's bits."""
    print(f"w4a16 small batch {m} x {n} x {k}, {waves} wavefronts, depth {depth}", flush=True)
    x16, codes, scales, zeros = _exact_case(900 + m + n + k, m, n, k)
    if k > 2048:
        scales[:] = np.float16(0.5)
    acc, _ = w4.product(x16, w4.dequant(codes, scales, zeros))
    acc32 = acc.astype(np.float32)
    assert np.array_equal(acc32.astype(np.float64), acc)
    pw, psz = _pack(codes, scales, zeros)
    rng = np.random.default_rng(16)
    mult = (1 + 0.25 * rng.standard_normal(n)).astype(np.float32)
    fbias = rng.standard_normal(n).astype(np.float32)
    o32, o16 = w4.epilogue_f32(acc32, mult, fbias)
    out = _forward(x16, pw, psz, n, None, None, torch.float32, waves=waves, depth=depth)
    np.testing.assert_array_equal(out.cpu().numpy(), acc32)
    outh = _forward(x16, pw, psz, n, mult, fbias, torch.float16, ldo=n + 24, waves=waves, depth=depth)
    np.testing.assert_array_equal(outh.cpu().numpy().view(np.uint16), o16.view(np.uint16))
    # bit-reproducible
    again = _forward(x16, pw, psz, n, None, None, torch.float32, waves=waves, depth=depth)
    assert torch.equal(out, again)


def test_small_batch_padded_activation_pitch(w4):
    m, n, k = 9, 256, 512
    x16, codes, scales, zeros = _exact_case(19, m, n, k)
    acc, _ = w4.product(x16, w4.dequant(codes, scales, zeros))
    pw, psz = _pack(codes, scales, zeros)
    xp = torch.zeros(m, k + 40, dtype=torch.float16, device=DEV)
    xp[:, :k] = _dev(x16)
    out = torch.empty(m, n, dtype=torch.float32, device=DEV)
    P.qlinear_w4a16_cwac_forward(xp[:, :k], pw, psz, n, None, None, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), acc.astype(np.float32))


@pytest.mark.parametrize("m,n,k", [(8, 512, 4096), (32, 12288, 4096), (16, 4096, 11008), (100, 512, 4096)])
def test_small_batch_workload_like(w4, m, n, k):
    """Decode-sized batches on LLM-like operands, up to the largest layer shapes of workload 5:
    every output inside the rounding bound of an fp32 summation of the exact products."""
    print(f"w4a16 small batch, workload-like {m} x {n} x {k}", flush=True)
    w, x16 = _llm_like(60 + k + m, m, n, k)
    codes, scales, zeros = w4.quantize_groupwise(w)
    wd = w4.dequant(codes, scales, zeros)
    acc, mag = w4.product(x16, wd)
    pw, psz = _pack(codes, scales, zeros)
    alpha = (1 + 0.05 * synth.normal(8, 0, n).numpy()).astype(np.float32)
    beta = (0.02 * synth.normal(8, 1, n).numpy()).astype(np.float32)
    mult, fbias = w4.fold(alpha, beta, None, n)
    ref = w4.folded_real(acc, mult, fbias)
    for dtype in (torch.float32, torch.float16):
        out = _forward(x16, pw, psz, n, mult, fbias, dtype).cpu().numpy().astype(np.float64)
        err = np.abs(out - ref)
        tol = _tolerance(mag, ref, k, mult, fbias, dtype == torch.float16)
        assert (err <= tol).all(), float((err / tol).max())
    out = _forward(x16, pw, psz, n, None, None, torch.float32).cpu().numpy().astype(np.float64)
    assert (np.abs(out - acc) <= 0.25 * _tolerance(mag, acc, k, None, None, False)).all()


def test_forward_longest_k(w4):
    """The largest supported K (256 quantization groups): every partial sum still exact in fp32."""
    m, n, k = 40, 256, 32768
    x16, codes, scales, zeros = _exact_case(77, m, n, k)
    scales[:] = np.float16(0.5)
    wd = w4.dequant(codes, scales, zeros)
    acc, _ = w4.product(x16, wd)
    assert np.abs(acc).max() < 2 ** 23
    pw, psz = _pack(codes, scales, zeros)
    out = _forward(x16, pw, psz, n, None, None, torch.float32)
    np.testing.assert_array_equal(out.cpu().numpy(), acc.astype(np.float32))


def test_forward_padded_activation_pitch(w4):
    m, n, k = 260, 256, 256
    x16, codes, scales, zeros = _exact_case(9, m, n, k)
    wd = w4.dequant(codes, scales, zeros)
    acc, _ = w4.product(x16, wd)
    pw, psz = _pack(codes, scales, zeros)
    xp = torch.zeros(m, k + 40, dtype=torch.float16, device=DEV)
    xp[:, :k] = _dev(x16)
    out = torch.empty(m, n, dtype=torch.float32, device=DEV)
    P.qlinear_w4a16_cwac_forward(xp[:, :k], pw, psz, n, None, None, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), acc.astype(np.float32))


# ------------------------------------------------------------------ forward: workload-like operands
def _tolerance(mag, ref, k, mult, fbias, half_out):
    mu = 1.0 if mult is None else np.abs(mult.astype(np.float64))[None, :]
    fb = 0.0 if fbias is None else np.abs(fbias.astype(np.float64))[None, :]
    tol = 8.0 * np.sqrt(k) * U * mag * mu + 4.0 * U * (np.abs(ref) + fb)
    if half_out:
        tol = tol + 2.0 ** -11 * np.abs(ref) + 2.0 ** -25
    return tol


def _llm_like(seed, m, n, k, n_outlier=3):
    w = (synth.normal(seed, 1, n * k).numpy() * 0.02).reshape(n, k)
    x = synth.normal(seed, 2, m * k).numpy().reshape(m, k).copy()
    ch = synth.uniform_ints(seed, 3, n_outlier, k)
    x[:, ch] *= 100.0 * np.exp(0.5 * synth.normal(seed, 4, n_outlier).numpy())
    return w.astype(np.float32), x.astype(np.float16)


@pytest.mark.parametrize("m,n,k", [(300, 512, 512), (640, 256, 4096)])
def test_forward_workload_like(w4, m, n, k):
    print(f"w4a16 workload-like {m} x {n} x {k}", flush=True)
    w, x16 = _llm_like(50 + k, m, n, k)
    codes, scales, zeros = w4.quantize_groupwise(w)
    wd = w4.dequant(codes, scales, zeros)
    acc, mag = w4.product(x16, wd)
    pw, psz = _pack(codes, scales, zeros)
    alpha = (1 + 0.05 * synth.normal(7, 0, n).numpy()).astype(np.float32)
    beta = (0.02 * synth.normal(7, 1, n).numpy()).astype(np.float32)
    mult, fbias = w4.fold(alpha, beta, None, n)
    ref = w4.folded_real(acc, mult, fbias)
    for pipe in w4_pipes(n, auto=False):
        for dtype in (torch.float32, torch.float16):
            out = _forward(x16, pw, psz, n, mult, fbias, dtype, pipe=pipe).cpu().numpy().astype(np.float64)
            err = np.abs(out - ref)
            tol = _tolerance(mag, ref, k, mult, fbias, dtype == torch.float16)
            assert (err <= tol).all(), float((err / tol).max())
        # the fp32 result sits far inside the bound: a dropped or misplaced term would not
        out = _forward(x16, pw, psz, n, None, None, torch.float32, pipe=pipe).cpu().numpy().astype(np.float64)
        assert (np.abs(out - acc) <= 8.0 * np.sqrt(k) * U * mag + 1e-30).all()
        assert np.abs(out - acc).max() <= 0.05 * (mag / k).mean()


def test_calibration_pipeline(w4, orc):
    """fp32 calibration forward -> statistics -> fit -> fold -> compensated binary16 forward."""
    n, k, rows = 512, 1024, 1536
    w, x16 = _llm_like(61, rows, n, k)
    codes0, scales0, zeros0 = w4.quantize_groupwise(w)
    wd = w4.dequant(codes0, scales0, zeros0)
    acc, mag = w4.product(x16, wd)
    y_full = (x16.astype(np.float64) @ w.astype(np.float64).T).astype(np.float32)
    alpha0, beta0 = orc.fit(y_full, acc.astype(np.float32))

    codes = torch.empty(n, k, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n, k // 128, dtype=torch.float16, device=DEV)
    zeros = torch.empty(n, k // 128, dtype=torch.uint8, device=DEV)
    P.cwac_w4_quantize_groupwise(_dev(w), codes, scales, zeros)
    pw = torch.empty(P.cwac_w4_packed_w_bytes(n, k), dtype=torch.uint8, device=DEV)
    psz = torch.empty((k // 128) * n, dtype=torch.int32, device=DEV)
    P.cwac_w4_pack(codes, scales, zeros, pw, psz)
    xd = _dev(x16)
    yq = torch.empty(rows, n, dtype=torch.float32, device=DEV)
    P.qlinear_w4a16_cwac_forward(xd, pw, psz, n, None, None, yq)
    st = torch.empty(P.cwac_stats_bytes(n) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, n)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(rows, n), dtype=torch.uint8, device=DEV)
    P.cwac_calibrate_stats(_dev(y_full), yq, st, ws)
    alpha = torch.empty(n, dtype=torch.float32, device=DEV)
    beta = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_solve(st, n, alpha, beta)
    mult = torch.empty(n, dtype=torch.float32, device=DEV)
    fbias = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_fold_weight_only(alpha, beta, None, mult, fbias)
    out = torch.empty(rows, n, dtype=torch.float16, device=DEV)
    P.qlinear_w4a16_cwac_forward(xd, pw, psz, n, mult, fbias, out)
    torch.cuda.synchronize()

    a, b = alpha.cpu().numpy(), beta.cpu().numpy()
    sf = y_full.astype(np.float64).std(axis=0)
    assert np.max(np.abs(a - alpha0) / np.maximum(np.abs(alpha0), 1.0)) <= 1e-5
    assert np.max(np.abs(b - beta0) / np.maximum(np.abs(beta0), sf)) <= 1e-5
    m0, f0 = w4.fold(a, b, None, n)
    np.testing.assert_array_equal(mult.cpu().numpy(), m0)
    np.testing.assert_array_equal(fbias.cpu().numpy(), f0)
    ref = w4.folded_real(acc, m0, f0)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    assert (err <= _tolerance(mag, ref, k, m0, f0, True)).all()
    # the compensation does what Sec. 3.3 fits it for
    e0 = ((acc - y_full) ** 2).sum()
    e1 = ((ref - y_full) ** 2).sum()
    assert e1 < e0


# ------------------------------------------------------------------ full layer sizes, sampled rows
def _sample_rows(m):
    rows = list(range(0, 4)) + list(range(254, 258)) + list(range(m - 4, m))
    rows += list(range(300, m - 300, max(1, (m - 600) // 12)))
    return np.unique(np.clip(np.array(rows, dtype=np.int64), 0, m - 1))


@pytest.mark.parametrize("layer", [1, 2, 4])
def test_full_size_llm_layers(w4, layer):
    """Workload 5's layer shapes in the benchmark's launch configuration; the oracle computes
    every output channel of a sample of token rows."""
    wl = synth.WORKLOADS[5]
    ly = wl.layers[layer]
    m, n, k = wl.m, ly.n, ly.k
    print(f"w4a16 full size {ly.name}: {m} x {n} x {k}", flush=True)
    w_d = synth.weights(wl, layer, device=DEV)[0]
    x_d = synth.activations(wl, layer, m, device=DEV).to(torch.float16)
    codes = torch.empty(n, k, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n, k // 128, dtype=torch.float16, device=DEV)
    zeros = torch.empty(n, k // 128, dtype=torch.uint8, device=DEV)
    P.cwac_w4_quantize_groupwise(w_d, codes, scales, zeros)
    pw = torch.empty(P.cwac_w4_packed_w_bytes(n, k), dtype=torch.uint8, device=DEV)
    psz = torch.empty((k // 128) * n, dtype=torch.int32, device=DEV)
    P.cwac_w4_pack(codes, scales, zeros, pw, psz)
    seed = wl.seed(layer) + 99
    alpha = (1.0 + 0.05 * synth.normal(seed, 0, n).numpy()).astype(np.float32)
    beta = (0.02 * synth.normal(seed, 1, n).numpy()).astype(np.float32)
    mult, fbias = w4.fold(alpha, beta, None, n)
    out = torch.empty(m, n, dtype=torch.float16, device=DEV)
    P.qlinear_w4a16_cwac_forward(x_d, pw, psz, n, _dev(mult), _dev(fbias), out)
    torch.cuda.synchronize()

    rows = _sample_rows(m)
    # the oracle dequantizes the device's codes (the quantizer's own parity is tested above) and
    # reads the activations the device used
    w_cpu = w_d.cpu().numpy()
    c0, s0, z0 = w4.quantize_groupwise(w_cpu)
    np.testing.assert_array_equal(codes.cpu().numpy(), c0)
    np.testing.assert_array_equal(scales.cpu().numpy().view(np.uint16), s0.view(np.uint16))
    wd = w4.dequant(c0, s0, z0)
    x_rows = x_d[torch.from_numpy(rows).to(DEV)].cpu().numpy()
    acc, mag = w4.product(x_rows, wd)
    ref = w4.folded_real(acc, mult, fbias)
    got = out[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    tol = _tolerance(mag, ref, k, mult, fbias, True)
    assert (err <= tol).all(), float((err / tol).max())
    # a prompt of 500 tokens on the same layer: the 128-token tile, at the launch shape it has there
    mh = 500
    out_h = torch.empty(mh, n, dtype=torch.float16, device=DEV)
    P.qlinear_w4a16_cwac_forward(x_d[:mh], pw, psz, n, _dev(mult), _dev(fbias), out_h)
    torch.cuda.synchronize()
    sel = np.nonzero(rows < mh)[0]
    got_h = out_h[torch.from_numpy(rows[sel]).to(DEV)].cpu().numpy().astype(np.float64)
    err_h = np.abs(got_h - ref[sel])
    assert (err_h <= tol[sel]).all(), float((err_h / tol[sel]).max())
