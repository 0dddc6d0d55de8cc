"""GPU parity of the calibration forward with the statistics fused into its epilogue
(qlinear_cwac_calibrate_fused): per-channel moments and (alpha, beta) against the fp64
oracle, which takes them from ITS OWN Y_quant (integer GEMM + dequantization) and the same
Y_full; and against the library's two-call path (fp32 forward, then cwac_calibrate_stats)."""
import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-5


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def _check_moments(mom, ref, rtol=RTOL):
    sf, sq = np.sqrt(ref[4]), np.sqrt(ref[2])
    floors = [sf, sq, sq * sq, sq * sf, sf * sf]
    for i in range(5):
        den = np.maximum(np.abs(ref[i]), floors[i]) + 1e-300
        err = np.abs(mom[i] - ref[i]) / den
        assert err.max() <= rtol, (i, err.max(), int(err.argmax()))


def _inputs(orc, seed, m, n, k, per_token, bias):
    g = synth.normal(seed, 0, m * k).numpy().reshape(m, k)
    xq = np.clip(np.rint(g * 50), -128, 127).astype(np.int8)
    g = synth.normal(seed, 1, n * k).numpy().reshape(n, k)
    wq = np.clip(np.rint(g * 45), -127, 127).astype(np.int8)
    mult = (np.abs(synth.normal(seed, 2, n).numpy()) * 2e-4 + 1e-4).astype(np.float32)
    off = np.rint(synth.normal(seed, 3, n).numpy() * 300).astype(np.int32)
    fb = synth.normal(seed, 4, n).numpy().astype(np.float32) if bias else None
    if bias:
        fb[5] = 3000.0          # a channel whose mean dwarfs its spread
        mult[5] = 1e-7
    sxr = (np.abs(synth.normal(seed, 5, m).numpy()) + 0.5).astype(np.float32) if per_token else None
    acc = orc.gemm_i8(xq, wq)
    _, yq = orc.folded_forward(acc, off, mult, 0, fb, sxr, want_f32=True)
    gain = (1.0 + 0.1 * synth.normal(seed, 6, n).numpy()).astype(np.float32)
    noise = synth.normal(seed, 7, m * n).numpy().reshape(m, n).astype(np.float32)
    yf = (yq * gain[None, :] + np.float32(0.05) * yq.std(axis=0, dtype=np.float64).astype(np.float32)[None, :]
          * noise + np.float32(0.01)).astype(np.float32)
    return xq, wq, mult, off, fb, sxr, yq, yf


def _solve(st, n):
    alpha = torch.empty(n, dtype=torch.float32, device=DEV)
    beta = torch.empty(n, dtype=torch.float32, device=DEV)
    mom = torch.empty(5, n, dtype=torch.float64, device=DEV)
    P.cwac_solve(st, n, alpha, beta, mom)
    return host(alpha), host(beta), host(mom)


def _new_state(n):
    st = torch.empty(P.cwac_stats_bytes(n) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, n)
    return st


def _fused(xq, wq, mult, off, fb, sxr, yf, st, waves=0):
    m, n = yf.shape
    ws = torch.empty(P.cwac_calibrate_fused_workspace(m, n), dtype=torch.uint8, device=DEV)
    P.qlinear_cwac_calibrate_fused(xq, wq, mult, off, fb, sxr, yf, st, ws,
                                   tuning=P.make_tuning(stats_waves=waves) if waves else None)


def _two_calls(xq, wq, mult, off, fb, sxr, yf, st):
    m, n = yf.shape
    yq = torch.empty(m, n, dtype=torch.float32, device=DEV)
    P.qlinear_cwac_forward(xq, wq, None, mult, off, fb, sxr, P.CWAC_OUT_FP32, yq)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(m, n), dtype=torch.uint8, device=DEV)
    P.cwac_calibrate_stats(yf, yq, st, ws)


@pytest.mark.parametrize("m,n,k,per_token,bias", [
    (256, 256, 128, False, False),      # exactly one tile
    (300, 520, 384, True, True),        # shifted edge tiles in both directions
    (700, 1028, 1152, False, True),     # several tiles, ragged tail of 188 rows / 4 channels
    (513, 768, 256, True, False),       # a last row tile that keeps a single row
])
@pytest.mark.parametrize("pipe", [None, "4w"])
def test_fused_calibration_against_oracle(orc, m, n, k, per_token, bias, pipe):
    """`pipe`: the default tile of eight wavefronts, or the four-wavefront shape of the same kernel."""
    print(f"fused calibration {m} x {n} x {k} per_token={per_token} bias={bias} pipe={pipe}", flush=True)
    waves = 4 if pipe == "4w" else 0
    xq, wq, mult, off, fb, sxr, yq, yf = _inputs(orc, 4100 + m, m, n, k, per_token, bias)
    ref = orc.channel_moments(yf, yq)
    a0, b0, _ = orc.solve(ref)
    d = [dev(v) for v in (xq, wq, mult, off, fb, sxr, yf)]
    st = _new_state(n)
    _fused(*d, st, waves)
    alpha, beta, mom = _solve(st, n)
    _check_moments(mom, ref)
    sf = np.sqrt(ref[4])
    assert np.max(np.abs(alpha - a0) / np.maximum(np.abs(a0), 1.0)) <= RTOL
    assert np.max(np.abs(beta - b0) / np.maximum(np.abs(b0), sf)) <= RTOL
    assert int(host(st.view(torch.int64)[:1])[0]) == m
    # the two-call path sees the same Y_quant: moments agree far below the parity bar
    st2 = _new_state(n)
    _two_calls(*d, st2)
    _, _, mom2 = _solve(st2, n)
    _check_moments(mom, mom2, rtol=1e-9)
    # bit-reproducible
    st3 = _new_state(n)
    _fused(*d, st3, waves)
    words = P.cwac_stats_bytes(n) // 8                   # the buffers carry spare words
    assert torch.equal(st[:words], st3[:words])


def test_fused_calibration_streams_batches(orc):
    """Three batches into one state, fused and two-call mixed: the moments are those of all rows."""
    m, n, k = 1100, 512, 256
    xq, wq, mult, off, fb, sxr, yq, yf = _inputs(orc, 4242, m, n, k, True, True)
    ref = orc.channel_moments(yf, yq)
    st = _new_state(n)
    cuts = [(0, 300), (300, 700), (700, 1100)]
    calls = [_fused, _two_calls, _fused]
    for (a, b), call in zip(cuts, calls):
        call(dev(xq[a:b]), dev(wq), dev(mult), dev(off), dev(fb), dev(sxr[a:b]), dev(yf[a:b]), st)
    _, _, mom = _solve(st, n)
    _check_moments(mom, ref)
    assert int(host(st.view(torch.int64)[:1])[0]) == m


def test_fused_calibration_rejects_unsupported_shapes():
    n, k = 256, 128
    wq = torch.zeros(n, k, dtype=torch.int8, device=DEV)
    mult = torch.ones(n, dtype=torch.float32, device=DEV)
    st = _new_state(n)
    for m in (1, 255):
        xq = torch.zeros(m, k, dtype=torch.int8, device=DEV)
        yf = torch.zeros(m, n, dtype=torch.float32, device=DEV)
        ws = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
        with pytest.raises(P.CwacError):
            P.qlinear_cwac_calibrate_fused(xq, wq, mult, None, None, None, yf, st, ws)
    xq = torch.zeros(256, k, dtype=torch.int8, device=DEV)
    yf = torch.zeros(256, n, dtype=torch.float32, device=DEV)
    with pytest.raises(P.CwacError):                     # workspace too small
        P.qlinear_cwac_calibrate_fused(xq, wq, mult, None, None, None, yf, st,
                                       torch.empty(64, dtype=torch.uint8, device=DEV))
    assert int(host(st.view(torch.int64)[:1])[0]) == 0   # nothing was accumulated


@pytest.mark.parametrize("cfg,layer", [(2, 0), (5, 1)])
def test_fused_calibration_full_size(orc, cfg, layer):
    """The benchmark's launch: one calibration batch of the workload's token count.  The oracle
    computes Y_quant and the moments for a sample of channels over ALL rows; every channel is
    checked against the library's two-call path."""
    wl = synth.WORKLOADS[cfg]
    ly = wl.layers[layer]
    m, n, k = wl.m, ly.n, ly.k
    print(f"config {cfg} layer {ly.name}: fused calibration {m} x {n} x {k}", flush=True)
    w_t, b_t = synth.weights(wl, layer, device=DEV)
    x_t = synth.activations(wl, layer, m, calibration=True, device=DEV)
    yf = x_t @ w_t.t()
    if b_t is not None:
        yf += b_t
    wq = torch.empty(n, k, dtype=torch.int8, device=DEV)
    sw = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_quantize_rows_sym(w_t, sw, wq)
    colsum = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_colsum(wq, colsum)
    xq = torch.empty(m, k, dtype=torch.int8, device=DEV)
    if wl.per_token:
        sxr = torch.empty(m, dtype=torch.float32, device=DEV)
        P.cwac_quantize_rows_sym(x_t, sxr, xq)
        sx, zx = 1.0, 0
    else:
        mm = torch.empty(2, dtype=torch.float32, device=DEV)
        ws = torch.empty(P.cwac_range_workspace(x_t.numel()), dtype=torch.uint8, device=DEV)
        P.cwac_range_f32(x_t, mm, ws)
        mn, mx = (float(v) for v in mm.cpu())
        sx, z_u = P.cwac_qparams_from_range(mn, mx, 8)
        zx = z_u - 128
        P.cwac_quantize_act(x_t, sx, zx, xq)
        sxr = None
    qpd = P.make_qparams(P.CWAC_EPI_FP_BIAS, wl.per_token, sx, zx, 1.0, 0)
    dm = torch.empty(n, dtype=torch.float32, device=DEV)
    do = torch.empty(n, dtype=torch.int32, device=DEV)
    dfb = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_fold(None, None, sw, b_t, colsum, qpd, dm, do, dfb)
    fb = dfb if b_t is not None else None
    st = _new_state(n)
    _fused(xq, wq, dm, do, fb, sxr, yf, st)
    alpha, beta, mom = _solve(st, n)
    st2 = _new_state(n)
    _two_calls(xq, wq, dm, do, fb, sxr, yf, st2)
    a2, b2, mom2 = _solve(st2, n)
    _check_moments(mom, mom2, rtol=1e-9)
    np.testing.assert_allclose(alpha, a2, rtol=1e-6, atol=1e-6)
    # oracle on sampled channels, all rows
    ch = np.unique(np.concatenate([np.arange(0, 8), np.arange(250, 262), np.arange(n - 8, n),
                                   np.arange(300, n - 300, max(1, (n - 600) // 24))]))
    xq_h, wq_h = host(xq), host(wq)[ch]
    acc = orc.gemm_i8(xq_h, wq_h)
    np.testing.assert_array_equal(host(wq)[ch], orc.quantize_rows_sym(host(w_t)[ch])[0])
    _, yq0 = orc.folded_forward(acc, host(do)[ch], host(dm)[ch], 0,
                                None if fb is None else host(fb)[ch],
                                None if sxr is None else host(sxr), want_f32=True)
    ref = orc.channel_moments(host(yf)[:, ch], yq0)
    _check_moments(mom[:, ch], ref)
    a0, b0, _ = orc.solve(ref)
    sf = np.sqrt(ref[4])
    assert np.max(np.abs(alpha[ch] - a0) / np.maximum(np.abs(a0), 1.0)) <= RTOL
    assert np.max(np.abs(beta[ch] - b0) / np.maximum(np.abs(b0), sf)) <= RTOL
