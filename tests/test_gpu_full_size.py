"""GPU parity at the workloads' full layer sizes, in the launch configuration the
benchmark times (automatic kernel choice, whole token batch).  The oracle checks
every output channel of a sample of token rows (first / last rows of the first
and last tiles plus a stride through the middle), which it can compute one by
one; statistics are checked over all rows of one calibration batch."""
import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

LAYERS = [(2, 0), (3, 0), (3, 1), (3, 2), (3, 3), (4, 0), (4, 1), (4, 2),
          (5, 0), (5, 1), (5, 2), (5, 4)]


def _sample_rows(m):
    rows = list(range(0, 8)) + list(range(250, 262)) + list(range(m - 8, m))
    rows += list(range(300, m - 300, max(1, (m - 600) // 20)))
    return np.unique(np.clip(np.array(rows, dtype=np.int64), 0, m - 1))


def _dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.mark.parametrize("cfg,layer", LAYERS)
def test_full_size_forward(orc, cfg, layer):
    _check_forward(orc, cfg, layer, synth.WORKLOADS[cfg].m)


@pytest.mark.parametrize("layer,m", [(0, 512), (1, 1024), (4, 1024), (1, 256)])
def test_llm_layers_few_tokens(orc, layer, m):
    """Workload 5's layer shapes at 256-1024 tokens: few tiles and a long K loop, where the automatic
    choice takes the 128 x 128 tile of the direct-to-LDS kernel (or small generic tiles)."""
    _check_forward(orc, 5, layer, m)


def _check_forward(orc, cfg, layer, m):
    wl = synth.WORKLOADS[cfg]
    ly = wl.layers[layer]
    n, k = ly.n, ly.k
    print(f"config {cfg} layer {ly.name}: {m} x {n} x {k}", flush=True)
    w_t, b_t = synth.weights(wl, layer)
    x_t = synth.activations(wl, layer, m)
    rows = _sample_rows(m)
    seed = wl.seed(layer) + 77
    alpha = (1.0 + 0.05 * synth.normal(seed, 0, n).numpy()).astype(np.float32)
    beta = (0.02 * synth.normal(seed, 1, n).numpy()).astype(np.float32)

    # ---- device: quantize, fold, forward (everything in the library's kernels)
    w_d, x_d = w_t.to(DEV), x_t.to(DEV)
    wq = torch.empty(n, k, dtype=torch.int8, device=DEV)
    sw = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_quantize_rows_sym(w_d, sw, wq)
    colsum = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_colsum(wq, colsum)
    xq = torch.empty(m, k, dtype=torch.int8, device=DEV)
    bias_d = None if b_t is None else b_t.to(DEV)
    if wl.per_token:
        sx_row = torch.empty(m, dtype=torch.float32, device=DEV)
        P.cwac_quantize_rows_sym(x_d, sx_row, xq)
        sx, zx = 1.0, 0
        mode = P.CWAC_EPI_FP_BIAS
    else:
        mm = torch.empty(2, dtype=torch.float32, device=DEV)
        ws = torch.empty(P.cwac_range_workspace(x_d.numel()), dtype=torch.uint8, device=DEV)
        P.cwac_range_f32(x_d, mm, ws)
        mn, mx = (float(v) for v in mm.cpu())
        sx, z_u = P.cwac_qparams_from_range(mn, mx, 8)
        zx = z_u - 128
        P.cwac_quantize_act(x_d, sx, zx, xq)
        sx_row = None
        mode = P.CWAC_EPI_INT_OFFSET
    # output scale: the layer output has a spread of about w_std * ||x_row||; aim at codes of spread ~30
    sr = float(np.float32(wl.w_std * np.linalg.norm(x_t.numpy()[rows], axis=1).mean() / 30.0))
    zr = 3
    qp = P.make_qparams(mode, wl.per_token, sx, zx, sr, zr)
    mult = torch.empty(n, dtype=torch.float32, device=DEV)
    off = torch.empty(n, dtype=torch.int32, device=DEV)
    fb = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_fold(_dev(alpha), _dev(beta), sw, bias_d, colsum, qp, mult, off, fb)
    out = torch.empty(m, n, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward(xq, wq, qp, mult, off, fb if wl.per_token else None, sx_row,
                           P.CWAC_OUT_INT8, out)
    # calibration forward (fp32 Y_quant) on the same batch
    qpd = P.make_qparams(P.CWAC_EPI_FP_BIAS, wl.per_token, sx, zx, 1.0, 0)
    dm = torch.empty(n, dtype=torch.float32, device=DEV)
    do = torch.empty(n, dtype=torch.int32, device=DEV)
    dfb = torch.empty(n, dtype=torch.float32, device=DEV)
    P.cwac_fold(None, None, sw, bias_d, colsum, qpd, dm, do, dfb)
    yq = torch.empty(m, n, dtype=torch.float32, device=DEV)
    P.qlinear_cwac_forward(xq, wq, None, dm, do, dfb if bias_d is not None else None, sx_row,
                           P.CWAC_OUT_FP32, yq)
    torch.cuda.synchronize()

    # ---- oracle on the sampled rows
    w, x = w_t.numpy(), x_t.numpy()
    bias = None if b_t is None else b_t.numpy()
    wq0, sw0 = orc.quantize_rows_sym(w)
    cs0 = orc.colsum_i8(wq0)
    np.testing.assert_array_equal(wq.cpu().numpy(), wq0)
    np.testing.assert_array_equal(sw.cpu().numpy(), sw0)
    np.testing.assert_array_equal(colsum.cpu().numpy(), cs0)
    if wl.per_token:
        xq0, sxr0 = orc.quantize_rows_sym(x[rows])
        np.testing.assert_array_equal(sx_row.cpu().numpy()[rows], sxr0)
        deq = sw0
        m0, fb0, o0 = orc.fold_fp_bias(alpha, beta, sw0, bias, cs0, True, 1.0, 0, sr)
    else:
        mn0, mx0 = orc.range_f32(x)
        s0, z0 = orc.qparams_asym(mn0, mx0, 8)
        assert (np.float32(sx), zx) == (s0, z0 - 128)
        xq0 = orc.quantize_act_i8(x[rows], s0, z0 - 128)
        sxr0 = None
        deq = orc.deq_scale(sw0, s0)
        m0, o0, _ = orc.fold_int_offset(alpha, beta, sw0, bias, cs0, s0, z0 - 128, sr)
        fb0 = None
    np.testing.assert_array_equal(xq.cpu().numpy()[rows], xq0)
    np.testing.assert_array_equal(mult.cpu().numpy(), m0)
    np.testing.assert_array_equal(off.cpu().numpy(), o0)
    acc = orc.gemm_i8(xq0, wq0)
    want = orc.folded_forward(acc, o0, m0, zr, fb0, sxr0)
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got[rows], want)
    assert 0.01 < np.mean(np.abs(want.astype(np.int32)) < 120), "codes should not all saturate"
    yq0 = orc.dequant_output(acc, cs0, zx, deq, bias, sxr0)
    np.testing.assert_array_equal(yq.cpu().numpy()[rows], yq0)
    # a property that holds at any size: plain-PTQ parameters through the same launch equal the
    # un-fused epilogue applied to the raw accumulators of the same launch shape
    acc_d = torch.empty(m, n, dtype=torch.int32, device=DEV)
    P.qlinear_cwac_forward(xq, wq, None, None, None, None, None, P.CWAC_OUT_INT32, acc_d)
    out2 = torch.empty(m, n, dtype=torch.int8, device=DEV)
    P.cwac_epilogue_int32(acc_d, qp, mult, off, fb if wl.per_token else None, sx_row,
                          P.CWAC_OUT_INT8, out2)
    assert torch.equal(out, out2)
    np.testing.assert_array_equal(acc_d.cpu().numpy()[rows], acc)


@pytest.mark.parametrize("cfg,layer", [(2, 0), (4, 2), (5, 0)])
def test_full_size_statistics(orc, cfg, layer):
    """One calibration batch of the benchmark's size (the workload's token count) through
    cwac_calibrate_stats + cwac_solve, all rows and channels against the fp64 oracle."""
    wl = synth.WORKLOADS[cfg]
    ly = wl.layers[layer]
    rows, c = wl.m, ly.n
    print(f"config {cfg} layer {ly.name}: statistics over {rows} x {c}", flush=True)
    seed = wl.seed(layer) + 99
    yq = synth.normal(seed, 0, rows * c).view(rows, c)
    yq[:, 5] = yq[:, 5] * 0.01 + 300.0                       # mean >> spread
    gain = 1.0 + 0.1 * synth.normal(seed, 1, c)
    yf = yq * gain[None, :] + 0.05 * synth.normal(seed, 2, rows * c).view(rows, c) + 0.01
    yq_d, yf_d = yq.to(DEV), yf.to(DEV)
    st = torch.empty(P.cwac_stats_bytes(c) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, c)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(rows, c), dtype=torch.uint8, device=DEV)
    P.cwac_calibrate_stats(yf_d, yq_d, st, ws)
    alpha = torch.empty(c, dtype=torch.float32, device=DEV)
    beta = torch.empty(c, dtype=torch.float32, device=DEV)
    mom = torch.empty(5, c, dtype=torch.float64, device=DEV)
    P.cwac_solve(st, c, alpha, beta, mom)
    torch.cuda.synchronize()
    ref = orc.channel_moments(yf.numpy(), yq.numpy())
    a0, b0, _ = orc.solve(ref)
    got = mom.cpu().numpy()
    sf, sq = np.sqrt(ref[4]), np.sqrt(ref[2])
    floors = [sf, sq, sq * sq, sq * sf, sf * sf]
    for i in range(5):
        err = np.abs(got[i] - ref[i]) / (np.maximum(np.abs(ref[i]), floors[i]) + 1e-300)
        assert err.max() <= 1e-5, (i, err.max())
    a, b = alpha.cpu().numpy(), beta.cpu().numpy()
    assert np.max(np.abs(a - a0) / np.maximum(np.abs(a0), 1.0)) <= 1e-5
    assert np.max(np.abs(b - b0) / np.maximum(np.abs(b0), sf)) <= 1e-5
