"""The whole calibration set of the LLM workload (128 x 2048 = 262144 rows) streamed into ONE
calibration state in 16 chunks of 16384 rows, as the benchmark's streaming leg does, for the
layer `o` (4096 x 4096): row count, moments and the fitted (alpha, beta) after the last chunk
against the fp64 oracle, which runs on the downloaded columns of a sample of channels (all rows);
the device's Y_quant of sampled rows is tied to the oracle bit for bit."""
import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-5


def test_full_calibration_set_streams_into_one_state(orc):
    wl = synth.WORKLOADS[5]
    li = 1
    ly = wl.layers[li]
    n, k, rows, chunk = ly.n, ly.k, wl.cal_rows, wl.m
    assert rows == 262144 and chunk == 16384 and rows % chunk == 0
    print(f"workload 5 layer {ly.name}: {rows} calibration rows in {rows // chunk} chunks, {n} channels", flush=True)
    f32 = dict(dtype=torch.float32, device=DEV)
    w = synth.weights(wl, li, device=DEV)[0]
    wq = torch.empty(n, k, dtype=torch.int8, device=DEV)
    sw = torch.empty(n, **f32)
    P.cwac_quantize_rows_sym(w, sw, wq)
    colsum = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_colsum(wq, colsum)
    dm, dfb = torch.empty(n, **f32), torch.empty(n, **f32)
    do = torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_fold(None, None, sw, None, colsum, P.make_qparams(P.CWAC_EPI_FP_BIAS, True, 1.0, 0, 1.0, 0), dm, do, dfb)

    rng = np.random.default_rng(5)
    ch = np.unique(np.concatenate([[0, 1, 255, 256, n - 1], rng.choice(n, 43, replace=False)]))
    ch_d = torch.from_numpy(ch).to(DEV)
    srows = np.unique(np.concatenate([[0, 1, chunk - 1, chunk, rows - 1], rng.choice(rows, 19, replace=False)]))
    yf_s = torch.empty(rows, len(ch), **f32)
    yq_s = torch.empty(rows, len(ch), **f32)
    x_rows, yq_rows = {}, {}

    st = torch.full((P.cwac_stats_bytes(n) // 8 + 2,), float("nan"), dtype=torch.float64, device=DEV)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(chunk, n), dtype=torch.uint8, device=DEV)
    xq = torch.empty(chunk, k, dtype=torch.int8, device=DEV)
    sx = torch.empty(chunk, **f32)
    yf = torch.empty(chunk, n, **f32)
    yq = torch.empty(chunk, n, **f32)
    for ci, c0 in enumerate(range(0, rows, chunk)):
        x = synth.activations(wl, li, chunk, calibration=True, device=DEV, row0=c0)
        P.cwac_quantize_rows_sym(x, sx, xq)
        torch.matmul(x, w.t(), out=yf)                         # the upstream full-precision layer
        P.qlinear_cwac_forward(xq, wq, None, dm, do, None, sx, P.CWAC_OUT_FP32, yq)
        P.cwac_calibrate_stats(yf, yq, st, ws, first=(ci == 0))
        yf_s[c0:c0 + chunk] = yf[:, ch_d]
        yq_s[c0:c0 + chunk] = yq[:, ch_d]
        for r in srows[(srows >= c0) & (srows < c0 + chunk)]:
            x_rows[int(r)] = x[int(r - c0)].cpu().numpy()
            yq_rows[int(r)] = yq[int(r - c0)].cpu().numpy()
    alpha, beta = torch.empty(n, **f32), torch.empty(n, **f32)
    mom = torch.empty(5, n, dtype=torch.float64, device=DEV)
    P.cwac_solve(st, n, alpha, beta, mom)
    torch.cuda.synchronize()
    assert int(st.view(torch.int64)[0].item()) == rows

    # the device's Y_quant rows are the oracle's, bit for bit (ties the streamed arrays to the oracle)
    wq0, sw0 = orc.quantize_rows_sym(w.cpu().numpy())
    cs0 = orc.colsum_i8(wq0)
    xs = np.stack([x_rows[int(r)] for r in srows])
    xq0, sx0 = orc.quantize_rows_sym(xs)
    yq0 = orc.dequant_output(orc.gemm_i8(xq0, wq0), cs0, 0, sw0, None, sx0)
    np.testing.assert_array_equal(np.stack([yq_rows[int(r)] for r in srows]), yq0)

    # moments and fit of the sampled channels over all 262144 rows
    ref = orc.channel_moments(yf_s.cpu().numpy(), yq_s.cpu().numpy())
    a0, b0, _ = orc.solve(ref)
    got = mom.cpu().numpy()[:, ch]
    sf, sq = np.sqrt(ref[4]), np.sqrt(ref[2])
    floors = [sf, sq, sq * sq, sq * sf, sf * sf]
    for i in range(5):
        err = np.abs(got[i] - ref[i]) / (np.maximum(np.abs(ref[i]), floors[i]) + 1e-300)
        assert err.max() <= RTOL, (i, err.max())
    a, b = alpha.cpu().numpy()[ch], beta.cpu().numpy()[ch]
    assert np.max(np.abs(a - a0) / np.maximum(np.abs(a0), 1.0)) <= RTOL
    assert np.max(np.abs(b - b0) / np.maximum(np.abs(b0), sf)) <= RTOL
