"""GPU parity on seeded random shapes: the dispatchers pick among many kernels and tile shapes by
size thresholds and divisibility; whatever they pick, integer results must equal the oracle's bit
for bit.  Every shape runs in the automatic choice and, where the direct-to-LDS kernel's
constraints hold, with that kernel forced."""

import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from tuning import tuning_of, w4_pipes

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _knobs(force_fast):
    """The kernel-choice override of a forward call: the direct-to-LDS kernel forced, or none."""
    return tuning_of("fast") if force_fast else None


def _linear_shapes():
    rng = np.random.default_rng(20250527)
    shapes = []
    for _ in range(28):
        shapes.append((int(rng.integers(1, 1400)), int(rng.integers(1, 700)), 16 * int(rng.integers(1, 80))))
    # around the dispatch thresholds: 256 rows, 128 / 256 channels, K multiples of 64 and 128
    shapes += [(255, 256, 128), (256, 127, 192), (257, 128, 64), (256, 255, 320), (511, 257, 448),
               (1025, 129, 1088), (300, 256, 80), (256, 384, 16)]
    return shapes


@pytest.mark.parametrize("m,n,k", _linear_shapes())
def test_linear_random_shape(orc, m, n, k):
    print(f"linear {m} x {n} x {k}", flush=True)
    rng = np.random.default_rng(m * 1000003 + n * 1009 + k)
    xq = rng.integers(-128, 128, (m, k), dtype=np.int8)
    wq = rng.integers(-127, 128, (n, k), dtype=np.int8)
    acc = orc.gemm_i8(xq, wq)
    mult = (np.abs(rng.standard_normal(n)) * 3e-4 + 1e-5).astype(np.float32)
    off = rng.integers(-5000, 5000, n).astype(np.int32)
    fb = rng.standard_normal(n).astype(np.float32)
    sxr = (np.abs(rng.standard_normal(m)) * 0.5 + 0.5).astype(np.float32)
    zr = int(rng.integers(-20, 20))
    qp = P.make_qparams(z_r=zr)
    qpt = P.make_qparams(P.CWAC_EPI_FP_BIAS, True, 1.0, 0, 1.0, zr)
    ldo = n + int(rng.integers(0, 3)) * 4
    # the automatic choice, the direct-to-LDS kernel forced, and its persistent tile on one to three
    # workgroups (every workgroup then walks several tiles; shapes it does not admit fall back)
    for tun in (None, tuning_of("fast"),
                tuning_of("fast", pipe="persist", persist_workgroups=int(rng.integers(1, 4)))):
        if True:
            def run(out_kind, dt, *args):
                full = torch.full((m, ldo), 55, dtype=dt, device=DEV)
                P.qlinear_cwac_forward(dev(xq), dev(wq), *args, out_kind, full[:, :n], tuning=tun)
                torch.cuda.synchronize()
                got = full.cpu().numpy()
                assert np.all(got[:, n:] == 55), "wrote outside the output columns"
                return got[:, :n]
            np.testing.assert_array_equal(
                run(P.CWAC_OUT_INT32, torch.int32, None, None, dev(off), None, None), acc + off[None, :])
            np.testing.assert_array_equal(
                run(P.CWAC_OUT_INT8, torch.int8, qp, dev(mult), dev(off), None, None),
                orc.folded_forward(acc, off, mult, zr))
            np.testing.assert_array_equal(
                run(P.CWAC_OUT_INT8, torch.int8, qp, dev(mult), dev(off), dev(fb), None),
                orc.folded_forward(acc, off, mult, zr, fb))
            np.testing.assert_array_equal(
                run(P.CWAC_OUT_INT8, torch.int8, qpt, dev(mult), dev(off), dev(fb), dev(sxr)),
                orc.folded_forward(acc, off, mult, zr, fb, sxr))
            _, want = orc.folded_forward(acc, off, mult, 0, fb, sxr, want_f32=True)
            np.testing.assert_array_equal(
                run(P.CWAC_OUT_FP32, torch.float32, None, dev(mult), dev(off), dev(fb), dev(sxr)), want)


def _conv_shapes():
    rng = np.random.default_rng(20250528)
    shapes = []
    for _ in range(14):
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        pad = int(rng.integers(0, min(kh, kw)))
        shapes.append((int(rng.integers(1, 7)), int(rng.integers(5, 21)), int(rng.integers(5, 21)),
                       16 * int(rng.integers(1, 13)), int(rng.integers(8, 300)), kh, kw,
                       int(rng.integers(1, 3)), pad))
    # shapes the direct-to-LDS kernel accepts (64 | c_in, 128 | K, >= 128 channels, >= 256 rows)
    shapes += [(3, 12, 12, 64, 130, 2, 2, 1, 0), (2, 16, 15, 128, 255, 3, 3, 1, 1), (5, 9, 9, 192, 256, 2, 2, 1, 1),
               (2, 20, 20, 64, 320, 4, 2, 2, 1)]
    return shapes


@pytest.mark.parametrize("shape", _conv_shapes())
def test_conv_random_shape(orc, shape):
    b, h, w, c, n, kh, kw, stride, pad = shape
    print(f"conv {shape}", flush=True)
    rng = np.random.default_rng(sum(shape) * 7919 + c)
    xq = rng.integers(-128, 128, (b, h, w, c), dtype=np.int8)
    wq = rng.integers(-127, 128, (n, kh, kw, c), dtype=np.int8)
    zx, zr = int(rng.integers(-128, 128)), int(rng.integers(-20, 20))
    acc = orc.conv2d_i8(xq, wq, stride, pad, zx)
    m = acc.shape[0]
    mult = (np.abs(rng.standard_normal(n)) * 3e-4 + 1e-5).astype(np.float32)
    off = rng.integers(-5000, 5000, n).astype(np.int32)
    fb = rng.standard_normal(n).astype(np.float32)
    qp = P.make_qparams(z_x=zx, z_r=zr)
    # the automatic choice, the direct-to-LDS kernel forced, and its persistent tile on one to three
    # workgroups (every workgroup then walks several tiles; shapes it does not admit fall back)
    for tun in (None, tuning_of("fast"),
                tuning_of("fast", pipe="persist", persist_workgroups=int(rng.integers(1, 4)))):
        if True:
            def run(out_kind, dt, *args):
                out = torch.empty(m, n, dtype=dt, device=DEV)
                P.qconv2d_cwac_forward(dev(xq), dev(wq), stride, pad, qp, *args, out_kind, out, tuning=tun)
                torch.cuda.synchronize()
                return out.cpu().numpy()
            np.testing.assert_array_equal(run(P.CWAC_OUT_INT32, torch.int32, None, dev(off), None), acc + off[None, :])
            np.testing.assert_array_equal(run(P.CWAC_OUT_INT8, torch.int8, dev(mult), dev(off), None),
                                          orc.folded_forward(acc, off, mult, zr))
            np.testing.assert_array_equal(run(P.CWAC_OUT_INT8, torch.int8, dev(mult), dev(off), dev(fb)),
                                          orc.folded_forward(acc, off, mult, zr, fb))
            _, want = orc.folded_forward(acc, off, mult, 0, fb, want_f32=True)
            np.testing.assert_array_equal(run(P.CWAC_OUT_FP32, torch.float32, dev(mult), dev(off), dev(fb)), want)


def _w4_shapes():
    rng = np.random.default_rng(20250529)
    shapes = [(int(rng.integers(1, 600)), 32 * int(rng.integers(8, 21)), 128 * int(rng.integers(1, 9)))
              for _ in range(10)]
    shapes += [(int(rng.integers(1, 33)), 32 * int(rng.integers(8, 21)), 128 * int(rng.integers(1, 12)))
               for _ in range(6)]            # decode-sized batches: the weight-streaming kernel
    # several passes of the weight-streaming kernel (7 and 5 passes, a last pass of 8 rows / 1 row), and shapes just
    # past the point where its estimated cost exceeds a tile's K loop
    return shapes + [(32, 256, 128), (33, 256, 128), (1, 288, 1408), (200, 256, 4096), (129, 288, 3072),
                     (130, 256, 1536), (256, 256, 2560)]


@pytest.mark.parametrize("m,n,k", _w4_shapes())
def test_weight_only_random_shape(m, n, k):
    """Operands whose every partial sum is exact in fp32 (small integers, power-of-two scales): any
    order of accumulation gives the oracle's bits."""
    from oracle import w4a16_oracle as w4
    w4.build()
    print(f"w4a16 {m} x {n} x {k}", flush=True)
    rng = np.random.default_rng(m * 7919 + n * 31 + k)
    x16 = rng.integers(-3, 4, (m, k)).astype(np.float16)
    codes = rng.integers(0, 16, (n, k), dtype=np.uint8)
    zeros = rng.integers(0, 16, (n, k // 128), dtype=np.uint8)
    scales = (2.0 ** rng.integers(-3, 4, (n, k // 128))).astype(np.float16)
    acc, _ = w4.product(x16, w4.dequant(codes, scales, zeros))
    acc32 = acc.astype(np.float32)
    assert np.array_equal(acc32.astype(np.float64), acc)
    mult = (1 + 0.25 * rng.standard_normal(n)).astype(np.float32)
    fbias = rng.standard_normal(n).astype(np.float32)
    o32, o16 = w4.epilogue_f32(acc32, mult, fbias)
    pw = torch.empty(P.cwac_w4_packed_w_bytes(n, k), dtype=torch.uint8, device=DEV)
    psz = torch.empty((k // 128) * n, dtype=torch.int32, device=DEV)
    P.cwac_w4_pack(dev(codes), dev(scales), dev(zeros), pw, psz)
    for pipe in w4_pipes(n):
        tun = tuning_of(w4_pipe=pipe)
        out = torch.empty(m, n, dtype=torch.float32, device=DEV)
        P.qlinear_w4a16_cwac_forward(dev(x16), pw, psz, n, dev(mult), dev(fbias), out, tuning=tun)
        outh = torch.empty(m, n, dtype=torch.float16, device=DEV)
        P.qlinear_w4a16_cwac_forward(dev(x16), pw, psz, n, dev(mult), dev(fbias), outh, tuning=tun)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy(), o32)
        np.testing.assert_array_equal(outh.cpu().numpy().view(np.uint16), o16.view(np.uint16))


# ------------------------------------------------------------------ Transformer-block glue
def _ln_shapes():
    rng = np.random.default_rng(77)
    shapes = [(int(rng.integers(1, 300)), 8 * int(rng.integers(1, 257))) for _ in range(16)]
    # channel counts on either side of the lanes-per-row choices (16, 32, 64 lanes x 1..4 vectors)
    return shapes + [(7, 8), (7, 128), (7, 136), (7, 384), (7, 392), (7, 512), (7, 520), (7, 768), (7, 776),
                     (7, 1024), (7, 1032), (7, 1536), (7, 1544), (7, 2048), (1, 640), (64, 16)]


@pytest.mark.parametrize("m,c", _ln_shapes())
def test_residual_ln_quant_random_shape(m, c):
    from oracle import block_oracle as blk
    print(f"residual + layer norm + quantizer {m} x {c}", flush=True)
    rng = np.random.default_rng(m * 4099 + c)
    h = (rng.standard_normal((m, c)) * 2).astype(np.float16)
    r = rng.integers(-128, 128, (m, c)).astype(np.int8)
    gamma = (1 + 0.2 * rng.standard_normal(c)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(c)).astype(np.float32)
    s_r, z_r, s_x, z_x = np.float32(0.02), -3, np.float32(0.025), 9
    h1 = torch.empty(m, c, dtype=torch.float16, device=DEV)
    xq = torch.empty(m, c, dtype=torch.int8, device=DEV)
    P.vit_residual_ln_quant(dev(h), dev(r), float(s_r), z_r, h1, dev(gamma), dev(beta), 1e-5, float(s_x), z_x, xq)
    torch.cuda.synchronize()
    want16, t = blk.residual(h, r, s_r, z_r)
    got16 = h1.cpu().numpy()
    slack = 2 * 2.0 ** -24 * (np.abs(h.astype(np.float64)) + np.abs(t)) + 1e-30
    g = got16.astype(np.float64)
    assert ((g >= (t - slack).astype(np.float16)) & (g <= (t + slack).astype(np.float16))).all()
    _, v = blk.quantize(blk.layernorm(g, gamma, beta, 1e-5), s_x, z_x)
    delta = 64 * 2.0 ** -24 * (np.abs(v) + 128) + 1e-4
    lo, hi = np.clip(np.rint(v - delta), -128, 127), np.clip(np.rint(v + delta), -128, 127)
    got = xq.cpu().numpy().astype(np.float64)
    assert ((got >= lo) & (got <= hi)).all()


def _attention_shapes():
    rng = np.random.default_rng(78)
    shapes = [(int(rng.integers(1, 4)), int(rng.integers(1, 225)), int(rng.integers(1, 5))) for _ in range(10)]
    long_ones = [(int(rng.integers(1, 3)), int(rng.integers(225, 900)), int(rng.integers(1, 3))) for _ in range(5)]
    return shapes + long_ones + [(1, 32, 1), (1, 31, 1), (1, 96, 1), (1, 97, 1), (1, 192, 1), (1, 223, 1), (2, 224, 2),
                                 (1, 672, 1), (1, 673, 1), (1, 257, 2)]


@pytest.mark.parametrize("with_bias", [False, True])
@pytest.mark.parametrize("head_dim", [64, 32])
@pytest.mark.parametrize("batch,tokens,heads", _attention_shapes())
def test_attention_random_shape(batch, tokens, heads, head_dim, with_bias):
    from oracle import block_oracle as blk
    print(f"attention {batch} x {tokens} x {heads} heads of {head_dim}, bias {with_bias}", flush=True)
    rng = np.random.default_rng(batch * 100000 + tokens * 100 + heads + head_dim)
    c = head_dim * heads
    r = np.clip(np.rint(rng.standard_normal((batch * tokens, 3 * c)) * 35 - 6), -128, 127).astype(np.int8)
    s, z = np.float32(0.035), -6
    bias = bias16 = None
    if with_bias:  # rows padded to whole key tiles plus a random surplus of 4-element steps
        ldb = 32 * ((tokens + 31) // 32) + 4 * int(rng.integers(0, 5))
        bias16 = np.full((heads, tokens, ldb), -77.0, dtype=np.float16)
        bias16[:, :, :tokens] = (rng.standard_normal((heads, tokens, tokens)) * 1.5).astype(np.float16)
        bias = bias16[:, :, :tokens].astype(np.float64)
    o, mag = blk.attention_codes(r, s, z, batch, tokens, heads, bias)
    s_a = np.float32(max(float(o.max() - o.min()), 1e-6) / 255.0)
    z_a = int(np.clip(round(-128 - float(o.min()) / float(s_a)), -128, 127))
    a = torch.empty(batch * tokens, c, dtype=torch.int8, device=DEV)
    P.vit_attention_int8(dev(r), float(s), z, batch, tokens, heads, float(s_a), z_a, a, head_dim=head_dim,
                         bias=None if bias16 is None else dev(bias16))
    torch.cuda.synchronize()
    _, v = blk.quantize(o, s_a, z_a)
    delta = (2.0 ** -11 + 1024 * 2.0 ** -24) * mag / s_a + 64 * 2.0 ** -24 * (np.abs(v) + 128) + 1e-4
    lo, hi = np.clip(np.rint(v - delta), -128, 127), np.clip(np.rint(v + delta), -128, 127)
    got = a.cpu().numpy().astype(np.float64)
    assert ((got >= lo) & (got <= hi)).all()
    assert (got == np.clip(np.rint(v), -128, 127)).mean() > 0.85
