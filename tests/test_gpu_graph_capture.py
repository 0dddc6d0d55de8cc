"""The whole step is capturable in a HIP graph: the library launches only kernels on the caller's
stream (no memset nodes, no allocation, no host synchronisation), so a captured step replays with
new input contents and gives what the eager calls give - checked on several replays with eager
work and synchronisations between them."""
import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_step_replays_from_a_graph(orc):
    wl = synth.WORKLOADS[1]
    m = cal = 512
    w_t, b_t = synth.weights(wl, 0, device=DEV)
    n, k = w_t.shape
    f32 = dict(dtype=torch.float32, device=DEV)
    i32 = dict(dtype=torch.int32, device=DEV)
    wq = torch.empty(n, k, dtype=torch.int8, device=DEV)
    sw = torch.empty(n, **f32)
    P.cwac_quantize_rows_sym(w_t, sw, wq)
    colsum = torch.empty(n, **i32)
    P.cwac_colsum(wq, colsum)
    sx, zx, sr, zr = 0.05, 3, 0.02, -5
    # static buffers of the captured step
    x = torch.empty(m, k, **f32)
    xcal = torch.empty(cal, k, **f32)
    yf = torch.empty(cal, n, **f32)
    xq = torch.empty(m, k, dtype=torch.int8, device=DEV)
    xqc = torch.empty(cal, k, dtype=torch.int8, device=DEV)
    dm, dfb, mult, fb = (torch.empty(n, **f32) for _ in range(4))
    do, off = torch.empty(n, **i32), torch.empty(n, **i32)
    alpha, beta = torch.empty(n, **f32), torch.empty(n, **f32)
    ndeg, nsat = torch.zeros(1, **i32), torch.zeros(1, **i32)
    yq = torch.empty(cal, n, **f32)
    st = torch.empty(P.cwac_stats_bytes(n) // 8 + 2, dtype=torch.float64, device=DEV)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(cal, n), dtype=torch.uint8, device=DEV)
    st_f = torch.empty_like(st)
    ws_f = torch.empty(P.cwac_calibrate_fused_workspace(cal, n), dtype=torch.uint8, device=DEV)
    alpha_f, beta_f = torch.empty(n, **f32), torch.empty(n, **f32)
    out = torch.empty(m, n, dtype=torch.int8, device=DEV)
    qpd = P.make_qparams(P.CWAC_EPI_FP_BIAS, False, sx, zx, 1.0, 0)
    qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, sx, zx, sr, zr)

    def step():
        P.cwac_quantize_act(x, sx, zx, xq)
        P.cwac_quantize_act(xcal, sx, zx, xqc)
        P.cwac_fold(None, None, sw, b_t, colsum, qpd, dm, do, dfb)
        P.qlinear_cwac_forward(xqc, wq, None, dm, do, dfb, None, P.CWAC_OUT_FP32, yq)
        P.cwac_stats_reset(st, n)
        P.cwac_calibrate_stats(yf, yq, st, ws)
        P.cwac_solve(st, n, alpha, beta, None, ndeg)
        P.cwac_fold(alpha, beta, sw, b_t, colsum, qp, mult, off, None, nsat)
        P.qlinear_cwac_forward(xq, wq, qp, mult, off, None, None, P.CWAC_OUT_INT8, out)
        P.cwac_stats_reset(st_f, n)                      # the one-call calibration side as well
        P.qlinear_cwac_calibrate_fused(xqc, wq, dm, do, dfb, None, yf, st_f, ws_f)
        P.cwac_solve(st_f, n, alpha_f, beta_f)

    def load(seed):
        x.copy_(synth.normal(seed, 0, m * k, device=DEV).view(m, k))
        xcal.copy_(synth.normal(seed, 1, cal * k, device=DEV).view(cal, k))
        yf.copy_(xcal @ w_t.t() + b_t)

    load(1)
    step()                                               # warm-up: one-time attribute calls
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for seed in (2, 3, 4):
        load(seed)
        step()                                           # eager reference on the same buffers
        torch.cuda.synchronize()
        want = [t.clone() for t in (out, alpha, beta, mult, off, alpha_f, beta_f, ndeg)]
        for t in (out, alpha, beta, mult, off, alpha_f, beta_f, yq, xq, xqc):
            t.zero_()                                    # eager work between the replays
        ndeg.fill_(7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, ref in zip((out, alpha, beta, mult, off, alpha_f, beta_f, ndeg), want):
            assert torch.equal(got, ref)
    # and the replayed result is the oracle's
    acc = orc.gemm_i8(xq.cpu().numpy(), wq.cpu().numpy())
    np.testing.assert_array_equal(out.cpu().numpy(),
                                  orc.folded_forward(acc, off.cpu().numpy(), mult.cpu().numpy(), zr))


def test_weight_only_and_convolution_replay_from_a_graph():
    """The weight-only INT4 entry points and the convolution launch only kernels too."""
    # the wide convolution below is too small for the dispatcher to pick the direct-to-LDS kernel
    lds = P.make_tuning(kernel=P.binding.CWAC_KERNEL_DIRECT_LDS)
    f32 = dict(dtype=torch.float32, device=DEV)
    m, n, k = 300, 512, 384
    w = synth.normal(3, 0, n * k, device=DEV).view(n, k) * 0.02
    x = torch.empty(m, k, dtype=torch.float16, device=DEV)
    codes = torch.empty(n, k, dtype=torch.uint8, device=DEV)
    sc = torch.empty(n, k // 128, dtype=torch.float16, device=DEV)
    ze = torch.empty(n, k // 128, dtype=torch.uint8, device=DEV)
    pw = torch.empty(P.cwac_w4_packed_w_bytes(n, k), dtype=torch.uint8, device=DEV)
    psz = torch.empty((k // 128) * n, dtype=torch.int32, device=DEV)
    alpha, beta = torch.empty(n, **f32), torch.empty(n, **f32)
    mult, fb = torch.empty(n, **f32), torch.empty(n, **f32)
    out = torch.empty(m, n, dtype=torch.float16, device=DEV)
    # convolution: 2 images of 12 x 12 x 32 -> 48 channels, 3 x 3, padding 1
    xc = torch.empty(2, 12, 12, 32, dtype=torch.int8, device=DEV)
    wc = torch.randint(-100, 101, (48, 3, 3, 32), dtype=torch.int8, device=DEV,
                       generator=torch.Generator(device=DEV).manual_seed(9))
    cm = torch.full((48,), 3e-4, **f32)
    co = torch.arange(48, dtype=torch.int32, device=DEV) * 7 - 100
    outc = torch.empty(2 * 12 * 12, 48, dtype=torch.int8, device=DEV)
    qp = P.make_qparams(z_x=-4, z_r=3)
    # the same weight-only layer at a decode-sized batch (the weight-streaming kernel) ...
    out8 = torch.empty(8, n, dtype=torch.float16, device=DEV)
    # ... and a convolution wide enough for the direct-to-LDS kernel: 4 images of 14 x 14 x 128 -> 256
    xw = torch.empty(4, 14, 14, 128, dtype=torch.int8, device=DEV)
    ww = torch.randint(-100, 101, (256, 3, 3, 128), dtype=torch.int8, device=DEV,
                       generator=torch.Generator(device=DEV).manual_seed(10))
    wm = torch.full((256,), 1e-4, **f32)
    wo = torch.arange(256, dtype=torch.int32, device=DEV) * 5 - 600
    outw = torch.empty(4 * 14 * 14, 256, dtype=torch.int8, device=DEV)

    def step():
        P.cwac_w4_quantize_groupwise(w, codes, sc, ze)
        P.cwac_w4_pack(codes, sc, ze, pw, psz)
        P.cwac_fold_weight_only(alpha, beta, None, mult, fb)
        P.qlinear_w4a16_cwac_forward(x, pw, psz, n, mult, fb, out)
        P.qlinear_w4a16_cwac_forward(x[:8], pw, psz, n, mult, fb, out8)
        P.qconv2d_cwac_forward(xc, wc, 1, 1, qp, cm, co, None, P.CWAC_OUT_INT8, outc, tuning=lds)
        P.qconv2d_cwac_forward(xw, ww, 1, 1, qp, wm, wo, None, P.CWAC_OUT_INT8, outw, tuning=lds)

    def load(seed):
        x.copy_(synth.normal(seed, 0, m * k, device=DEV).view(m, k))
        alpha.copy_(1.0 + 0.1 * synth.normal(seed, 1, n, device=DEV))
        beta.copy_(0.05 * synth.normal(seed, 2, n, device=DEV))
        xc.copy_((synth.normal(seed, 3, xc.numel(), device=DEV) * 40).clamp(-128, 127).view(xc.shape))
        xw.copy_((synth.normal(seed, 4, xw.numel(), device=DEV) * 40).clamp(-128, 127).view(xw.shape))

    load(1)
    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for seed in (2, 3, 4):
        load(seed)
        step()
        torch.cuda.synchronize()
        want = [t.clone() for t in (out, outc, mult, fb, out8, outw)]
        for t in (out, outc, mult, fb, pw, out8, outw):
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (out, outc, mult, fb, out8, outw)):
            assert torch.equal(a, b), f"replay {seed} differs from the eager step"


def test_transformer_block_replays_from_a_graph():
    """vit_block_w8a8_forward is kernel launches and nothing else."""
    import vit_block_fixture as vit_block
    batch, tokens, heads, hidden = 4, 50, 2, 256
    blk = vit_block.build_block(9, batch, tokens, heads, hidden, device=DEV)
    h = vit_block.residual_stream(9, blk.m, blk.c, DEV)
    h_out = torch.empty_like(h)
    ws = torch.empty(P.vit_block_workspace(batch, tokens, heads, hidden), dtype=torch.int8, device=DEV)
    P.vit_block_w8a8_forward(blk.params, h, h_out, ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        P.vit_block_w8a8_forward(blk.params, h, h_out, ws)
    for seed in (10, 11, 12):
        h.copy_(vit_block.residual_stream(seed, blk.m, blk.c, DEV))
        P.vit_block_w8a8_forward(blk.params, h, h_out, ws)
        torch.cuda.synchronize()
        want, want_ws = h_out.clone(), ws.clone()
        h_out.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(want, h_out) and torch.equal(want_ws, ws), f"replay {seed} differs from the eager call"
