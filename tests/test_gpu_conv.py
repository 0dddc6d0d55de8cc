"""GPU parity of the quantized convolutional layer with the CWAC epilogue (implicit GEMM on the
int8 matrix cores) against the CPU oracle, bit for bit, through the C ABI."""
from types import SimpleNamespace

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


def _conv(xq, wq, stride, pad, qp, out_kind, mult=None, offset=None, fbias=None, tile=None, ldo=None,
          pipe=None):
    b, h, w, _ = xq.shape
    n, kh, kw, _ = wq.shape
    oh, ow = (h + 2 * pad - kh) // stride + 1, (w + 2 * pad - kw) // stride + 1
    dt = {0: torch.int8, 1: torch.float32, 2: torch.int32}[out_kind]
    full = torch.full((b * oh * ow, ldo or n), 77, dtype=dt, device=DEV)
    view = full[:, :n]
    P.qconv2d_cwac_forward(dev(xq), dev(wq), stride, pad, qp, dev(mult), dev(offset), dev(fbias),
                           out_kind, view, tuning=tuning_of(tile, pipe))
    torch.cuda.synchronize()
    got = full.cpu().numpy()
    if ldo:
        assert np.all(got[:, n:] == 77), "wrote outside the output columns"
    return got[:, :n]


SHAPES = [  # batch, h, w, c_in, c_out, k, stride, pad
    (2, 14, 14, 64, 64, 3, 1, 1),      # ResNet-style 3x3
    (3, 15, 13, 32, 48, 3, 2, 1),      # stride 2, odd sizes
    (2, 9, 11, 128, 40, 1, 1, 0),      # pointwise
    (1, 23, 21, 16, 24, 7, 2, 3),      # stem-like 7x7 / 2
    (2, 8, 8, 16, 260, 3, 1, 0),       # no padding, channel edge of every tile shape
    (5, 7, 7, 48, 32, 1, 2, 0),        # strided pointwise (down-sampling shortcut)
]


@pytest.mark.parametrize("tile", [64, 128, 256])
@pytest.mark.parametrize("shape", SHAPES)
def test_conv_all_modes(orc, shape, tile):
    b, h, w, c, n, k, stride, pad = shape
    print(f"conv {shape} tile {tile}", flush=True)
    seed = 500 + h * 31 + c
    xq = np.clip(np.rint(synth.normal(seed, 0, b * h * w * c).numpy() * 50), -128, 127).astype(np.int8)
    xq = xq.reshape(b, h, w, c)
    wq = np.clip(np.rint(synth.normal(seed, 1, n * k * k * c).numpy() * 50), -127, 127).astype(np.int8)
    wq = wq.reshape(n, k, k, c)
    zx, zr = -11, 4
    acc = orc.conv2d_i8(xq, wq, stride, pad, zx)
    colsum = orc.colsum_i8(wq.reshape(n, -1))
    mult = (np.abs(synth.normal(seed, 2, n).numpy()) * 1e-3 + 1e-4).astype(np.float32)
    off = (np.rint(synth.normal(seed, 3, n).numpy() * 300).astype(np.int64) - zx * colsum).astype(np.int32)
    fb = synth.normal(seed, 4, n).numpy().astype(np.float32)
    qp = P.make_qparams(z_x=zx, z_r=zr)
    ldo = n + 3 if tile == 128 else None
    got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_INT32, tile=tile, ldo=ldo)
    np.testing.assert_array_equal(got, acc)
    got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_INT8, mult, off, tile=tile, ldo=ldo)
    np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, zr))
    got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_INT8, mult, off, fbias=fb, tile=tile, ldo=ldo)
    np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, zr, fb))
    _, want = orc.folded_forward(acc, off, mult, 0, fb, want_f32=True)
    got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_FP32, mult, off, fbias=fb, tile=tile, ldo=ldo)
    np.testing.assert_array_equal(got, want)


FAST_SHAPES = [  # batch, h, w, c_in, c_out, kh, kw, stride, pad, pipes
    (2, 14, 14, 128, 256, 3, 3, 1, 1, ("8w", "duo", "q")),  # ResNet-style 3x3, row tiles that overlap
    (5, 12, 11, 64, 300, 4, 4, 1, 2, ("duo",)),           # 64 channels: one K step per tap; ragged channel edge
    (2, 23, 21, 128, 256, 7, 7, 2, 3, ("8w", "duo", "q")),  # 7x7 / 2 with padding 3: most taps of the border rows are outside
    (3, 10, 16, 256, 260, 3, 5, 1, 2, ("8w", "duo")),     # rectangular filter, two K steps per tap
    (24, 9, 7, 128, 256, 3, 3, 2, 0, ("8w",)),            # stride 2 without padding
    (2, 14, 14, 128, 128, 3, 3, 1, 1, ("duo",)),          # fewer than 256 output channels: the 256 x 128 tile
    (3, 11, 13, 64, 176, 2, 2, 1, 1, ("duo",)),           # ... with overlapping channel tiles, 64 channels per tap
    (4, 14, 14, 64, 64, 3, 3, 1, 1, ("duo",)),            # 64 output channels: the 256 x 64 tile; K = 576
    (8, 12, 12, 128, 96, 3, 3, 2, 1, ("duo",)),           # ... overlapping 64-channel tiles, stride 2
]


@pytest.mark.parametrize("shape", FAST_SHAPES)
def test_conv_direct_to_lds_kernel(orc, shape):
    """The large-layer kernel (forced) as an implicit-GEMM convolution, in both tile shapes: padding
    taps come from a table of constant codes, every stage of K lies inside one filter tap."""
    b, h, w, c, n, kh, kw, stride, pad, pipes = shape
    seed = 900 + h * 31 + c + kh
    xq = np.clip(np.rint(synth.normal(seed, 0, b * h * w * c).numpy() * 50), -128, 127).astype(np.int8)
    xq = xq.reshape(b, h, w, c)
    wq = np.clip(np.rint(synth.normal(seed, 1, n * kh * kw * c).numpy() * 50), -127, 127).astype(np.int8)
    wq = wq.reshape(n, kh, kw, c)
    zx, zr = 9, -3
    acc = orc.conv2d_i8(xq, wq, stride, pad, zx)
    assert acc.shape[0] >= 256
    colsum = orc.colsum_i8(wq.reshape(n, -1))
    mult = (np.abs(synth.normal(seed, 2, n).numpy()) * 3e-4 + 1e-5).astype(np.float32)
    off = (np.rint(synth.normal(seed, 3, n).numpy() * 300).astype(np.int64) - zx * colsum).astype(np.int32)
    fb = synth.normal(seed, 4, n).numpy().astype(np.float32)
    qp = P.make_qparams(z_x=zx, z_r=zr)
    for pipe in pipes:
        print(f"conv {shape[:9]} direct-to-LDS kernel, pipe {pipe}", flush=True)
        kw_ = dict(tile="fast", pipe=pipe, ldo=n + 16 if pipe == "duo" else None)
        got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_INT32, **kw_)
        np.testing.assert_array_equal(got, acc)
        got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_INT8, mult, off, **kw_)
        np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, zr))
        got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_INT8, mult, off, fbias=fb, **kw_)
        np.testing.assert_array_equal(got, orc.folded_forward(acc, off, mult, zr, fb))
        _, want = orc.folded_forward(acc, off, mult, 0, fb, want_f32=True)
        got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_FP32, mult, off, fbias=fb, **kw_)
        np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("kh,kw,pad", [(1, 7, 0), (7, 1, 0), (3, 5, 2), (5, 3, 1)])
def test_conv_rectangular_filters(orc, kh, kw, pad):
    b, h, w, c, n = 3, 17, 19, 32, 72
    xq = np.clip(np.rint(synth.normal(60 + kh, 0, b * h * w * c).numpy() * 50), -128, 127).astype(np.int8)
    xq = xq.reshape(b, h, w, c)
    wq = np.clip(np.rint(synth.normal(60 + kh, 1, n * kh * kw * c).numpy() * 50), -127, 127).astype(np.int8)
    wq = wq.reshape(n, kh, kw, c)
    qp = P.make_qparams(z_x=9)
    for stride in (1, 2):
        got = _conv(xq, wq, stride, pad, qp, P.CWAC_OUT_INT32)
        np.testing.assert_array_equal(got, orc.conv2d_i8(xq, wq, stride, pad, 9))


def test_conv_pointwise_equals_linear(orc):
    """A 1x1 stride-1 convolution is the linear layer on the flattened positions."""
    b, h, w, c, n = 4, 16, 16, 256, 512
    xq = np.clip(np.rint(synth.normal(7, 0, b * h * w * c).numpy() * 40), -128, 127).astype(np.int8)
    wq = np.clip(np.rint(synth.normal(7, 1, n * c).numpy() * 40), -127, 127).astype(np.int8)
    qp = P.make_qparams(z_x=3)
    got = _conv(xq.reshape(b, h, w, c), wq.reshape(n, 1, 1, c), 1, 0, qp, P.CWAC_OUT_INT32)
    lin = torch.empty(b * h * w, n, dtype=torch.int32, device=DEV)
    P.qlinear_cwac_forward(dev(xq.reshape(-1, c)), dev(wq.reshape(n, c)), None, None, None, None, None,
                           P.CWAC_OUT_INT32, lin)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got, lin.cpu().numpy())


def test_conv_calibration_pipeline(orc):
    """fp32 layer -> quantizers -> calibration forward (fp32 out) -> statistics -> fit -> fold ->
    compensated int8 forward, every stage against the oracle."""
    b, h, w, c, n, k, stride, pad = 6, 14, 14, 64, 96, 3, 1, 1
    wf = (synth.normal(91, 0, n * k * k * c).numpy() * 0.05).reshape(n, k * k * c)
    bias = (synth.normal(91, 1, n).numpy() * 0.05).astype(np.float32)
    xf = np.maximum(synth.normal(91, 2, b * h * w * c).numpy(), 0.0).reshape(b, h, w, c)   # post-ReLU
    xf[..., 5] *= 12.0
    wq, sw = orc.quantize_rows_sym(wf)
    colsum = orc.colsum_i8(wq)
    mn, mx = orc.range_f32(xf)
    sx, z_u = orc.qparams_asym(mn, mx, 8)
    zx = z_u - 128
    xq = orc.quantize_act_i8(xf, sx, zx)
    wq4 = wq.reshape(n, k, k, c)
    acc = orc.conv2d_i8(xq, wq4, stride, pad, zx)
    deq = orc.deq_scale(sw, sx)
    y_quant = orc.dequant_output(acc, colsum, zx, deq, bias)
    # upstream full-precision layer: fp32 convolution through padded windows
    xp = np.zeros((b, h + 2, w + 2, c), dtype=np.float32)
    xp[:, 1:-1, 1:-1] = xf
    win = np.lib.stride_tricks.sliding_window_view(xp, (k, k), axis=(1, 2))
    y_full = (np.einsum("bhwcij,nijc->bhwn", win, wf.reshape(n, k, k, c).astype(np.float32))
              .reshape(-1, n) + bias).astype(np.float32)
    alpha, beta = orc.fit(y_full, y_quant)
    yc = orc.cwac_apply(y_quant, alpha, beta)
    sr, zr_u = orc.qparams_asym(*orc.range_f32(yc), 8)
    zr = zr_u - 128
    mult, offset, _ = orc.fold_int_offset(alpha, beta, sw, bias, colsum, sx, zx, sr)
    want = orc.folded_forward(acc, offset, mult, zr)

    f32 = dict(dtype=torch.float32, device=DEV)
    d_mult, d_fb = torch.empty(n, **f32), torch.empty(n, **f32)
    d_off = torch.empty(n, dtype=torch.int32, device=DEV)
    d_sw, d_bias, d_cs = dev(sw), dev(bias), torch.empty(n, dtype=torch.int32, device=DEV)
    P.cwac_colsum(dev(wq), d_cs)
    np.testing.assert_array_equal(d_cs.cpu().numpy(), colsum)
    qp_deq = P.make_qparams(P.CWAC_EPI_FP_BIAS, False, sx, zx, 1.0, 0)
    P.cwac_fold(None, None, d_sw, d_bias, d_cs, qp_deq, d_mult, d_off, d_fb)
    m = acc.shape[0]
    yq = torch.empty(m, n, **f32)
    P.qconv2d_cwac_forward(dev(xq), dev(wq4), stride, pad, qp_deq, d_mult, d_off, d_fb, P.CWAC_OUT_FP32, yq)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(yq.cpu().numpy(), y_quant)
    st = torch.empty(P.cwac_stats_bytes(n) // 8 + 2, dtype=torch.float64, device=DEV)
    P.cwac_stats_reset(st, n)
    ws = torch.empty(P.cwac_calibrate_stats_workspace(m, n), dtype=torch.uint8, device=DEV)
    P.cwac_calibrate_stats(dev(y_full), yq, st, ws)
    d_alpha, d_beta = torch.empty(n, **f32), torch.empty(n, **f32)
    P.cwac_solve(st, n, d_alpha, d_beta)
    torch.cuda.synchronize()
    a, be = d_alpha.cpu().numpy(), d_beta.cpu().numpy()
    sf = y_full.astype(np.float64).std(axis=0)
    assert np.max(np.abs(a - alpha) / np.maximum(np.abs(alpha), 1.0)) <= 1e-5
    assert np.max(np.abs(be - beta) / np.maximum(np.abs(beta), sf)) <= 1e-5
    qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, sx, zx, sr, zr)
    P.cwac_fold(dev(alpha), dev(beta), d_sw, d_bias, d_cs, qp, d_mult, d_off)
    np.testing.assert_array_equal(d_mult.cpu().numpy(), mult)
    np.testing.assert_array_equal(d_off.cpu().numpy(), offset)
    out = torch.empty(m, n, dtype=torch.int8, device=DEV)
    P.qconv2d_cwac_forward(dev(xq), dev(wq4), stride, pad, qp, d_mult, d_off, None, P.CWAC_OUT_INT8, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("b,h,c,n", [(64, 14, 256, 256), (128, 14, 256, 256), (32, 28, 128, 128),
                                     (8, 56, 64, 64), (128, 7, 512, 512)])
def test_conv_large_layer_sampled(orc, b, h, c, n):
    """ResNet-50-sized 3x3 layers (M = 12544 / 25088, K = 2304; M = 25088, N = 128, K = 1152; M = 25088,
    N = 64, K = 576; M = 6272, N = 512, K = 4608) in the automatic kernel choice (the generic kernel / the
    direct-to-LDS kernel in its 128 x 256, 256 x 128, 256 x 64 and 128 x 128 tiles); the oracle checks whole
    images (first, last) position by position."""
    w, k = h, 3
    xq = torch.randint(-128, 128, (b, h, w, c), dtype=torch.int8, device=DEV,
                       generator=torch.Generator(device=DEV).manual_seed(5))
    wq = torch.randint(-127, 128, (n, k, k, c), dtype=torch.int8, device=DEV,
                       generator=torch.Generator(device=DEV).manual_seed(6))
    qp = P.make_qparams(z_x=-5, z_r=2)
    mult = (np.abs(synth.normal(8, 2, n).numpy()) * 2e-4 + 1e-5).astype(np.float32)
    off = np.rint(synth.normal(8, 3, n).numpy() * 3000).astype(np.int32)
    out = torch.empty(b * h * w, n, dtype=torch.int8, device=DEV)
    P.qconv2d_cwac_forward(xq, wq, 1, 1, qp, dev(mult), dev(off), None, P.CWAC_OUT_INT8, out)
    torch.cuda.synchronize()
    xh, wh = xq.cpu().numpy(), wq.cpu().numpy()
    for img in (0, b - 1):
        acc = orc.conv2d_i8(xh[img:img + 1], wh, 1, 1, -5)
        want = orc.folded_forward(acc, off, mult, 2)
        np.testing.assert_array_equal(out[img * h * w:(img + 1) * h * w].cpu().numpy(), want)
