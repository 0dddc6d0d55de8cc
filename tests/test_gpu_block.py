"""GPU parity of the Transformer-block glue (residual + layer norm + quantizer, GELU table,
multi-head self-attention on int8 codes) against oracle/block_oracle.py, through the C ABI.

Where fp32 arithmetic decides an int8 code, the oracle supplies the real number v whose rounding is
the code and the test derives a bound `delta` on what the kernel's fp32 (attention: binary16
weights) evaluation can be off by; the kernel's code must be the rounding of some number in
[v - delta, v + delta] - exact wherever v is farther than delta from a tie."""
import math

import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from oracle import block_oracle as blk

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
U32 = 2.0 ** -24


def _dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _codes_within(got, v, delta, qmin=-128, qmax=127):
    lo = np.clip(np.rint(v - delta), qmin, qmax)
    hi = np.clip(np.rint(v + delta), qmin, qmax)
    g = got.astype(np.float64)
    bad = (g < lo) | (g > hi)
    assert not bad.any(), (int(bad.sum()), float(np.abs(g - np.clip(np.rint(v), qmin, qmax)).max()))
    return float((lo == hi).mean())  # share of outputs the check pins to one code


# ------------------------------------------------------------------ residual + layer norm + quantizer
def _ln_case(seed, m, c):
    rng = np.random.default_rng(seed)
    h = (rng.standard_normal((m, c)) * (1 + 4 * (rng.random(c) < 0.02))).astype(np.float16)
    r = rng.integers(-128, 128, (m, c)).astype(np.int8)
    gamma = (1 + 0.2 * rng.standard_normal(c)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(c)).astype(np.float32)
    return h, r, gamma, beta


@pytest.mark.parametrize("m,c", [(5, 64), (197, 768), (33, 1024), (10, 2048), (64, 384), (3, 8), (9, 1280)])
@pytest.mark.parametrize("with_residual", [False, True])
def test_residual_ln_quant(m, c, with_residual):
    print(f"residual + layer norm + quantizer {m} x {c}, residual {with_residual}", flush=True)
    h, r, gamma, beta = _ln_case(11 + m + c, m, c)
    s_r, z_r, eps = 0.01, 3, 1e-6
    # pitches wider than the row, outputs pre-filled: nothing outside the row may be written
    hp = torch.zeros(m, c + 8, dtype=torch.float16, device=DEV)
    hp[:, :c] = _dev(h)
    hout_full = torch.full((m, c + 16), 7.0, dtype=torch.float16, device=DEV)
    xq_full = torch.full((m, c + 8), 77, dtype=torch.int8, device=DEV)
    h_out = hout_full[:, :c] if with_residual else None
    r_d = _dev(r) if with_residual else None
    P.vit_residual_ln_quant(hp[:, :c], r_d, s_r, z_r, h_out, _dev(gamma), _dev(beta), eps, 0.03, -5,
                            xq_full[:, :c])
    torch.cuda.synchronize()
    assert (xq_full[:, c:] == 77).all() and (hout_full[:, c:] == 7.0).all()
    if with_residual:
        want16, t = blk.residual(h, r, s_r, z_r)
        got16 = h_out.cpu().numpy()
        # one fp32 product and one fp32 sum before the rounding to binary16
        slack = 2 * U32 * (np.abs(h.astype(np.float64)) + np.abs(t)) + 1e-30
        lo = (t - slack).astype(np.float16).astype(np.float64)
        hi = (t + slack).astype(np.float16).astype(np.float64)
        g = got16.astype(np.float64)
        assert ((g >= lo) & (g <= hi)).all()
        assert (got16 == want16).mean() > 0.999
        ln_in = got16.astype(np.float64)  # the layer norm reads the stored binary16 value
    else:
        assert (hout_full == 7.0).all()
        ln_in = h.astype(np.float64)
    y = blk.layernorm(ln_in, gamma, beta, eps)
    _, v = blk.quantize(y, 0.03, -5)
    # fp32: the two row sums (relative error ~ log2(c) u each), a handful of roundings per element
    delta = 64 * U32 * (np.abs(v) + 128) + 1e-4
    pinned = _codes_within(xq_full[:, :c].cpu().numpy(), v, delta)
    assert pinned > 0.99


def test_residual_only_and_quantizer_saturation():
    m, c = 6, 128
    h, r, gamma, beta = _ln_case(5, m, c)
    out = torch.empty(m, c, dtype=torch.float16, device=DEV)
    P.vit_residual_ln_quant(_dev(h), _dev(r), 0.5, -1, out, None, None, 0.0, 1.0, 0, None)
    torch.cuda.synchronize()
    want, _ = blk.residual(h, r, 0.5, -1)  # h + 0.5 * integer: exact in fp32, one rounding to binary16
    np.testing.assert_array_equal(out.cpu().numpy().view(np.uint16), want.view(np.uint16))
    # a tiny scale saturates the codes at both ends
    xq = torch.empty(m, c, dtype=torch.int8, device=DEV)
    P.vit_residual_ln_quant(_dev(h), None, 0.0, 0, None, _dev(gamma), _dev(beta), 1e-6, 1e-4, 0, xq)
    torch.cuda.synchronize()
    y = blk.layernorm(h.astype(np.float64), gamma, beta, 1e-6)
    sat = np.abs(y) > 0.02
    np.testing.assert_array_equal(xq.cpu().numpy()[sat], np.where(y[sat] > 0, 127, -128))


# ------------------------------------------------------------------ GELU table
@pytest.mark.parametrize("s_in,z_in,s_out,z_out", [(0.05, -20, 0.02, -120), (0.013, 7, 0.011, -113),
                                                   (0.2, 0, 0.1, -128), (1e-3, -128, 1e-3, -128)])
def test_gelu_table(s_in, z_in, s_out, z_out):
    tab = torch.empty(256, dtype=torch.int8, device=DEV)
    P.vit_gelu_table(s_in, z_in, s_out, z_out, tab)
    torch.cuda.synchronize()
    # the scales reach the kernel as fp32
    want, v = blk.gelu_table(np.float32(s_in), z_in, np.float32(s_out), z_out)
    got = tab.cpu().numpy()
    tie = np.abs(v - np.floor(v) - 0.5) < 1e-9
    np.testing.assert_array_equal(got[~tie], want[~tie])
    assert np.abs(got.astype(int) - want.astype(int)).max() <= 1


@pytest.mark.parametrize("m,n,pad", [(1, 16, 0), (197, 3072, 0), (33, 48, 16), (1000, 1536, 32)])
def test_table_lookup(m, n, pad):
    rng = np.random.default_rng(m + n)
    x = rng.integers(-128, 128, (m, n)).astype(np.int8)
    tab = rng.integers(-128, 128, 256).astype(np.int8)
    xp = torch.zeros(m, n + pad, dtype=torch.int8, device=DEV)
    xp[:, :n] = _dev(x)
    full = torch.full((m, n + pad), 55, dtype=torch.int8, device=DEV)
    P.vit_table_lookup(xp[:, :n], _dev(tab), full[:, :n])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(full[:, :n].cpu().numpy(), tab[x.astype(int) + 128])
    assert (full[:, n:] == 55).all()
    # in place
    P.vit_table_lookup(xp[:, :n], _dev(tab), xp[:, :n])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(xp[:, :n].cpu().numpy(), tab[x.astype(int) + 128])


# ------------------------------------------------------------------ attention
def _attention(r, s, z, batch, tokens, heads, s_a, z_a, pad=0):
    c = 64 * heads
    rp = torch.zeros(batch * tokens, 3 * c + pad, dtype=torch.int8, device=DEV)
    rp[:, :3 * c] = _dev(r)
    full = torch.full((batch * tokens, c + 2 * pad), 99, dtype=torch.int8, device=DEV)
    P.vit_attention_int8(rp[:, :3 * c], s, z, batch, tokens, heads, s_a, z_a, full[:, :c])
    torch.cuda.synchronize()
    assert (full[:, c:] == 99).all()
    return full[:, :c].cpu().numpy()


def _out_params(o):
    lo, hi = float(o.min()), float(o.max())
    s_a = np.float32(max(hi - lo, 1e-6) / 255.0)
    z_a = int(np.clip(round(-128 - lo / float(s_a)), -128, 127))
    return float(s_a), z_a


@pytest.mark.parametrize("batch,tokens,heads", [(2, 197, 3), (1, 224, 1), (3, 49, 2), (2, 1, 1), (1, 33, 2),
                                                (1, 64, 1), (2, 100, 12), (1, 193, 2)])
def test_attention_random_codes(batch, tokens, heads):
    print(f"attention {batch} x {tokens} tokens x {heads} heads", flush=True)
    rng = np.random.default_rng(batch * 1000 + tokens * 10 + heads)
    c = 64 * heads
    r = np.clip(np.rint(rng.standard_normal((batch * tokens, 3 * c)) * 30 + 4), -128, 127).astype(np.int8)
    s, z = np.float32(0.04), 4
    o, mag = blk.attention_codes(r, s, z, batch, tokens, heads)
    s_a, z_a = _out_params(o)
    got = _attention(r, float(s), z, batch, tokens, heads, s_a, z_a, pad=16)
    _, v = blk.quantize(o, np.float32(s_a), z_a)
    # weights rounded to binary16 (2^-11 relative, per term); fp32 exponent arguments of size up to a few
    # hundred (absolute error ~1e-5 in the exponent), fp32 exp2 / sums / normalization
    delta = (2.0 ** -11 + 1024 * U32) * mag / s_a + 64 * U32 * (np.abs(v) + 128) + 1e-4
    pinned = _codes_within(got, v, delta)
    want, _ = blk.quantize(o, np.float32(s_a), z_a)
    assert (got == want).mean() > 0.9, float((got == want).mean())
    print(f"  pinned to one code: {pinned:.3f}, equal to the oracle's code: {(got == want).mean():.4f}", flush=True)


@pytest.mark.parametrize("batch,tokens,heads,head_dim", [(6, 49, 4, 32), (2, 197, 2, 64), (3, 64, 1, 32),
                                                         (5, 20, 3, 64), (1, 224, 1, 32)])
def test_attention_with_logit_bias(batch, tokens, heads, head_dim):
    """A relative-position-like bias per head (binary16, rows padded to whole key tiles), shared by all images,
    with a few masked (very negative) entries."""
    print(f"attention with bias {batch} x {tokens} x {heads} heads of {head_dim}", flush=True)
    rng = np.random.default_rng(batch + 10 * tokens + heads + head_dim)
    c = head_dim * heads
    r = np.clip(np.rint(rng.standard_normal((batch * tokens, 3 * c)) * 30 + 4), -128, 127).astype(np.int8)
    s, z = np.float32(0.04), 4
    ldb = 32 * ((tokens + 31) // 32)
    bias16 = np.full((heads, tokens, ldb), 123.0, dtype=np.float16)          # padding: read, never used
    bias16[:, :, :tokens] = (rng.standard_normal((heads, tokens, tokens)) * 2).astype(np.float16)
    masked = rng.random((heads, tokens, tokens)) < 0.05
    masked[:, np.arange(tokens), np.arange(tokens)] = False                  # every query keeps a key
    bias16[:, :, :tokens][masked] = np.float16(-100.0)
    bias = bias16[:, :, :tokens].astype(np.float64)
    o, mag = blk.attention_codes(r, s, z, batch, tokens, heads, bias)
    s_a, z_a = _out_params(o)
    a = torch.empty(batch * tokens, c, dtype=torch.int8, device=DEV)
    P.vit_attention_int8(_dev(r), float(s), z, batch, tokens, heads, s_a, z_a, a, head_dim=head_dim,
                         bias=_dev(bias16))
    torch.cuda.synchronize()
    _, v = blk.quantize(o, np.float32(s_a), z_a)
    delta = (2.0 ** -11 + 1024 * U32) * mag / s_a + 64 * U32 * (np.abs(v) + 128) + 1e-4
    got = a.cpu().numpy()
    _codes_within(got, v, delta)
    want, _ = blk.quantize(o, np.float32(s_a), z_a)
    assert (got == want).mean() > 0.9
    # the bias matters: without it the codes differ
    o0, _ = blk.attention_codes(r, s, z, batch, tokens, heads)
    w0, _ = blk.quantize(o0, np.float32(s_a), z_a)
    assert (w0 != want).mean() > 0.2


@pytest.mark.parametrize("batch,tokens,heads,head_dim,with_bias", [
    (2, 225, 2, 64, False), (1, 448, 1, 64, False), (1, 449, 2, 32, False), (2, 577, 3, 64, False),
    (1, 1000, 2, 64, True), (1, 577, 2, 32, True), (1, 300, 1, 64, True), (1, 4096, 1, 64, False)])
def test_attention_long_sequences(batch, tokens, heads, head_dim, with_bias):
    """More than 224 tokens: the keys pass through the workgroup in chunks and the queries split into blocks
    of 224 - chunk counts 2 .. 19, last chunks of 1 token up to a full one, last query blocks ragged."""
    print(f"attention {batch} x {tokens} tokens x {heads} heads of {head_dim}, bias {with_bias}", flush=True)
    rng = np.random.default_rng(batch * 7 + tokens + heads + head_dim)
    c = head_dim * heads
    r = np.clip(np.rint(rng.standard_normal((batch * tokens, 3 * c)) * 30 + 4), -128, 127).astype(np.int8)
    s, z = np.float32(0.04), 4
    bias = bias16 = None
    if with_bias:
        ldb = 32 * ((tokens + 31) // 32)
        bias16 = np.full((heads, tokens, ldb), 123.0, dtype=np.float16)
        bias16[:, :, :tokens] = (rng.standard_normal((heads, tokens, tokens)) * 2).astype(np.float16)
        masked = rng.random((heads, tokens, tokens)) < 0.05
        masked[:, np.arange(tokens), np.arange(tokens)] = False
        bias16[:, :, :tokens][masked] = np.float16(-100.0)
        bias = bias16[:, :, :tokens].astype(np.float64)
    o, mag = blk.attention_codes(r, s, z, batch, tokens, heads, bias)
    s_a, z_a = _out_params(o)
    full = torch.full((batch * tokens, c + 16), 99, dtype=torch.int8, device=DEV)
    P.vit_attention_int8(_dev(r), float(s), z, batch, tokens, heads, s_a, z_a, full[:, :c], head_dim=head_dim,
                         bias=None if bias16 is None else _dev(bias16))
    torch.cuda.synchronize()
    assert (full[:, c:] == 99).all()
    got = full[:, :c].cpu().numpy()
    _, v = blk.quantize(o, np.float32(s_a), z_a)
    delta = (2.0 ** -11 + 1024 * U32) * mag / s_a + 64 * U32 * (np.abs(v) + 128) + 1e-4
    _codes_within(got, v, delta)
    want, _ = blk.quantize(o, np.float32(s_a), z_a)
    assert (got == want).mean() > 0.9, float((got == want).mean())


@pytest.mark.parametrize("tokens", [77, 500])
def test_attention_uniform_weights_is_the_mean_value(tokens):
    """All keys of a head equal: every weight is exactly 1 / tokens, the output is the mean value row -
    sharp in the layout of V, the head split, the masking of the padded keys and the normalization."""
    batch, heads = 2, 2
    c = 64 * heads
    rng = np.random.default_rng(3)
    r = rng.integers(-128, 128, (batch * tokens, 3 * c)).astype(np.int8)
    kk = rng.integers(-128, 128, (batch, 1, c)).astype(np.int8)
    r[:, c:2 * c] = np.broadcast_to(kk, (batch, tokens, c)).reshape(batch * tokens, c)
    s, z = np.float32(0.02), -9
    o, mag = blk.attention_codes(r, s, z, batch, tokens, heads)
    vmean = blk.dequantize(r[:, 2 * c:], s, z).reshape(batch, tokens, c).mean(axis=1)
    np.testing.assert_allclose(o.reshape(batch, tokens, c), np.broadcast_to(vmean[:, None, :], (batch, tokens, c)),
                               rtol=1e-12, atol=1e-12)
    s_a, z_a = _out_params(o)
    got = _attention(r, float(s), z, batch, tokens, heads, s_a, z_a)
    _, v = blk.quantize(o, np.float32(s_a), z_a)
    pinned = _codes_within(got, v, 64 * U32 * (np.abs(v) + 128 + mag / s_a) + 1e-4)
    assert pinned > 0.99


@pytest.mark.parametrize("tokens", [197, 600])
def test_attention_one_dominant_key_picks_its_value(tokens):
    """Query i scores key perm[i] far above the rest: the output row is that key's value row - sharp in
    which key's weight meets which value row (the key order of the second product)."""
    batch, heads = 1, 1
    c = 64
    rng = np.random.default_rng(4)
    perm = rng.permutation(tokens)
    # keys: distinct +-1 patterns scaled to +-100; query i = key perm[i]: score 64 * 100^2 against at most ~0.6 of it
    pat = rng.choice([-100, 100], size=(tokens, c))
    r = np.zeros((tokens, 3 * c), dtype=np.int8)
    r[:, c:2 * c] = pat
    r[:, :c] = pat[perm]
    r[:, 2 * c:] = rng.integers(-128, 128, (tokens, c))
    s, z = np.float32(0.05), 0
    o, mag = blk.attention_codes(r, s, z, batch, tokens, heads)
    vsel = blk.dequantize(r[perm, 2 * c:], s, z)
    np.testing.assert_allclose(o, vsel, atol=1e-9)
    s_a, z_a = float(s), 0
    got = _attention(r, float(s), z, batch, tokens, heads, s_a, z_a)
    np.testing.assert_array_equal(got, r[perm, 2 * c:])


def test_attention_row_subset_of_a_batch_matches_single_image():
    """Images are independent: image 1 of a batch of 3 equals the same image alone."""
    tokens, heads = 60, 2
    c = 64 * heads
    rng = np.random.default_rng(8)
    r = np.clip(np.rint(rng.standard_normal((3 * tokens, 3 * c)) * 25), -128, 127).astype(np.int8)
    a3 = _attention(r, 0.05, 1, 3, tokens, heads, 0.03, -2)
    a1 = _attention(r[tokens:2 * tokens], 0.05, 1, 1, tokens, heads, 0.03, -2)
    np.testing.assert_array_equal(a3[tokens:2 * tokens], a1)


# ------------------------------------------------------------------ the whole block
def _check_block_stages(orc, bk, h, t, rows):
    """Every stage of the staged run against the oracle, each fed the device's own previous output,
    on the token rows `rows` (attention: on the images those rows belong to)."""
    L = bk.layers
    tok = bk.tokens
    cpu = {k: v.cpu().numpy() for k, v in t.items()}
    h_np = h.cpu().numpy()
    ln = [x.cpu().numpy() for x in bk.ln]
    d_ln = lambda v: 64 * U32 * (np.abs(v) + 128) + 1e-4  # noqa: E731

    # x1 = Q(LN1(h))
    _, v = blk.quantize(blk.layernorm(h_np[rows], ln[0], ln[1], bk.eps), L[0]["s_x"], L[0]["z_x"])
    assert _codes_within(cpu["x1"][rows], v, d_ln(v)) > 0.99
    # the four linear layers: fold and folded forward of the main oracle, bit-exact
    for i, (x, r) in enumerate((("x1", "r1"), ("a", "r2"), ("x2", "r3"), ("g", "r4"))):
        ly = L[i]
        mult, offset, _ = orc.fold_int_offset(ly["alpha"].cpu().numpy(), ly["beta"].cpu().numpy(),
                                              ly["s_w"].cpu().numpy(), ly["bias"].cpu().numpy(),
                                              ly["colsum"].cpu().numpy(), ly["s_x"], ly["z_x"], ly["s_r"])
        np.testing.assert_array_equal(ly["mult"].cpu().numpy(), mult)
        np.testing.assert_array_equal(ly["offset"].cpu().numpy(), offset)
        acc = orc.gemm_i8(cpu[x], ly["w_q"].cpu().numpy(), rows=rows)
        np.testing.assert_array_equal(cpu[r][rows], orc.folded_forward(acc, offset, mult, ly["z_r"]))
    # attention on the images of the sampled rows
    images = np.unique(rows // tok)
    for b in images:
        sl = slice(b * tok, (b + 1) * tok)
        bias = None if bk.attn_bias is None else bk.attn_bias.cpu().numpy()[:, :, :tok].astype(np.float64)
        o, mag = blk.attention_codes(cpu["r1"][sl], np.float32(L[0]["s_r"]), L[0]["z_r"], 1, tok, bk.heads, bias)
        s_a = np.float32(L[1]["s_x"])
        _, v = blk.quantize(o, s_a, L[1]["z_x"])
        delta = (2.0 ** -11 + 1024 * U32) * mag / s_a + 64 * U32 * (np.abs(v) + 128) + 1e-4
        _codes_within(cpu["a"][sl], v, delta)
    # h1 = RN16(h + deq(r2)), x2 = Q(LN2(h1))
    want16, tt = blk.residual(h_np[rows], cpu["r2"][rows], np.float32(L[1]["s_r"]), L[1]["z_r"])
    slack = 2 * U32 * (np.abs(h_np[rows].astype(np.float64)) + np.abs(tt)) + 1e-30
    g16 = cpu["h1"][rows].astype(np.float64)
    assert ((g16 >= (tt - slack).astype(np.float16)) & (g16 <= (tt + slack).astype(np.float16))).all()
    _, v = blk.quantize(blk.layernorm(cpu["h1"][rows], ln[2], ln[3], bk.eps), L[2]["s_x"], L[2]["z_x"])
    assert _codes_within(cpu["x2"][rows], v, d_ln(v)) > 0.99
    # g = table[r3]
    want_tab, v = blk.gelu_table(np.float32(L[2]["s_r"]), L[2]["z_r"], np.float32(L[3]["s_x"]), L[3]["z_x"])
    got_tab = bk.gelu_table.cpu().numpy()
    tie = np.abs(v - np.floor(v) - 0.5) < 1e-9
    np.testing.assert_array_equal(got_tab[~tie], want_tab[~tie])
    np.testing.assert_array_equal(cpu["g"][rows], got_tab[cpu["r3"][rows].astype(int) + 128])
    # h2 = RN16(h1 + deq(r4))
    _, tt = blk.residual(cpu["h1"][rows], cpu["r4"][rows], np.float32(L[3]["s_r"]), L[3]["z_r"])
    slack = 2 * U32 * (np.abs(cpu["h1"][rows].astype(np.float64)) + np.abs(tt)) + 1e-30
    g16 = cpu["h2"][rows].astype(np.float64)
    assert ((g16 >= (tt - slack).astype(np.float16)) & (g16 <= (tt + slack).astype(np.float16))).all()


def _run_block(orc, seed, batch, tokens, heads, hidden, rows, head_dim=64, attn_bias=None):
    import vit_block_fixture as vit_block
    b = vit_block.build_block(seed, batch, tokens, heads, hidden, device=DEV, head_dim=head_dim,
                              attn_bias=None if attn_bias is None else _dev(attn_bias))
    h = vit_block.residual_stream(seed, b.m, b.c, DEV)
    t = vit_block.staged_forward(b, h)
    ws = torch.empty(P.vit_block_workspace(batch, tokens, heads, hidden), dtype=torch.int8, device=DEV)
    h_out = torch.empty_like(h)
    P.vit_block_w8a8_forward(b.params, h, h_out, ws)
    torch.cuda.synchronize()
    # the chained entry point computes the same steps: bit-identical results, documented workspace
    m, c = b.m, b.c
    assert torch.equal(h_out, t["h2"])
    assert torch.equal(ws[:m * c].view(m, c), t["x2"])
    assert torch.equal(ws[m * c:4 * m * c].view(m, 3 * c), t["r1"])
    assert torch.equal(ws[4 * m * c:5 * m * c].view(m, c), t["r4"])
    assert torch.equal(ws[5 * m * c:5 * m * c + m * hidden].view(m, hidden), t["g"])
    # the codes use their ranges (a block whose tensors saturate or collapse would test nothing)
    for k in ("x1", "r1", "a", "r2", "x2", "r3", "g", "r4"):
        codes = t[k].cpu().numpy()
        assert np.unique(codes).size > 60, (k, np.unique(codes).size)
    _check_block_stages(orc, b, h, t, rows)
    return b, t


def test_block_chain_small(orc):
    print("block: 3 images x 197 tokens, 3 heads, MLP 768", flush=True)
    _run_block(orc, 3, 3, 197, 3, 768, np.arange(3 * 197))


def test_block_chain_other_shapes(orc):
    print("block: 5 images x 50 tokens, 2 heads, MLP 256", flush=True)
    _run_block(orc, 4, 5, 50, 2, 256, np.arange(250))


@pytest.mark.parametrize("heads,hidden,name", [(6, 1536, "ViT-S"), (16, 4096, "ViT-L"), (20, 5120, "ViT-H")])
def test_block_other_model_widths(orc, heads, hidden, name):
    print(f"block: {name}, 2 images x 197 tokens, {heads} heads, MLP {hidden}", flush=True)
    _run_block(orc, 7 + heads, 2, 197, heads, hidden, np.arange(0, 394, 3))


def test_block_windowed_model_shapes(orc):
    """Swin-B stage 3: windows of 49 tokens as the attending units, 16 heads of 32, C = 512, MLP 2048, a
    relative-position-like bias per head on the logits."""
    print("block: 64 windows x 49 tokens, 16 heads of 32, MLP 2048, attention bias", flush=True)
    rng = np.random.default_rng(31)
    bias = np.zeros((16, 49, 64), dtype=np.float16)
    bias[:, :, :49] = rng.standard_normal((16, 49, 49)).astype(np.float16)
    _run_block(orc, 31, 64, 49, 16, 2048, np.arange(0, 64 * 49, 5), head_dim=32, attn_bias=bias)
    _run_block(orc, 32, 16, 49, 16, 2048, np.arange(0, 16 * 49, 3), head_dim=32)


def test_block_long_sequence(orc):
    """ViT-B/16 at 384 x 384 pixels: 577 tokens per image, attention over key chunks."""
    print("block: 2 images x 577 tokens, 12 heads, MLP 3072", flush=True)
    _run_block(orc, 9, 2, 577, 12, 3072, np.arange(0, 2 * 577, 2))


def test_block_full_size_sampled(orc):
    """ViT-B/16: 128 images x 197 tokens, 12 heads, MLP 3072 - the launch configuration the benchmark's
    block section times; the oracle checks three images' rows."""
    print("block: 128 images x 197 tokens, 12 heads, MLP 3072", flush=True)
    rows = np.concatenate([np.arange(0, 197), np.arange(63 * 197, 64 * 197), np.arange(127 * 197, 128 * 197)])
    _run_block(orc, 5, 128, 197, 12, 3072, rows)


def test_encoder_stack_equals_block_by_block():
    """Three blocks in one call (the residual of one block and the LN1 + quantizer of the next in one pass)
    against three single-block calls; then the same in place over the residual stream."""
    import vit_block_fixture as vit_block
    batch, tokens, heads, hidden = 6, 197, 3, 768
    blocks = [vit_block.build_block(20 + i, batch, tokens, heads, hidden, device=DEV) for i in range(3)]
    h = vit_block.residual_stream(20, batch * tokens, 64 * heads, DEV)
    ws = torch.empty(P.vit_block_workspace(batch, tokens, heads, hidden), dtype=torch.int8, device=DEV)
    a, b = h.clone(), torch.empty_like(h)
    for blk_ in blocks:
        P.vit_block_w8a8_forward(blk_.params, a, b, ws)
        a, b = b, a
    torch.cuda.synchronize()
    want = a.clone()
    assert not torch.equal(want, h)
    out = torch.empty_like(h)
    P.vit_encoder_w8a8_forward([x.params for x in blocks], h, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    inplace = h.clone()
    P.vit_encoder_w8a8_forward([x.params for x in blocks], inplace, inplace, ws)
    torch.cuda.synchronize()
    assert torch.equal(inplace, want)
    # blocks of different shapes do not stack
    other = vit_block.build_block(30, batch, tokens, heads, 512, device=DEV)
    with pytest.raises(P.CwacError):
        P.vit_encoder_w8a8_forward([blocks[0].params, other.params], h, out, ws)


def test_block_argument_errors():
    import vit_block_fixture as vit_block
    b = vit_block.build_block(6, 1, 16, 1, 64, device=DEV)
    h = vit_block.residual_stream(6, 16, 64, DEV)
    ws = torch.empty(P.vit_block_workspace(1, 16, 1, 64), dtype=torch.int8, device=DEV)
    with pytest.raises(P.CwacError):
        P.vit_block_w8a8_forward(b.params, h, torch.empty_like(h), ws[:100])


# ------------------------------------------------------------------ forward with a code table in its epilogue
@pytest.mark.parametrize("m,n,k,force", [
    (4096, 3072, 768, False),     # fused, 128-token tile pairs
    (16384, 1024, 1024, False),   # fused, 256-token tile
    (20001, 768, 768, False),     # fused, ragged last row tile
    (9000, 2048, 192, False),     # fused, K a multiple of 64 only
    (25216, 3072, 768, False),    # fused, persistent tile, 4.6 rounds of tiles
    (300, 256, 128, False),       # too small: forward, then a lookup pass in place
    (1000, 48, 64, False),        # narrow: two passes
    (256, 256, 64, True), (1000, 512, 192, True), (777, 1024, 128, True), (513, 272, 256, True),
])
def test_forward_with_code_table(m, n, k, force):
    """out = table[forward + 128], bit for bit, against the plain forward (itself checked against the
    oracle in test_gpu_parity.py) followed by numpy indexing."""
    print(f"forward with code table {m} x {n} x {k}, forced {force}", flush=True)
    rng = np.random.default_rng(m + n + k)
    x = torch.from_numpy(rng.integers(-128, 128, (m, k)).astype(np.int8)).to(DEV)
    w = torch.from_numpy(rng.integers(-127, 128, (n, k)).astype(np.int8)).to(DEV)
    mult = torch.from_numpy((rng.uniform(0.5, 1.5, n) * 40.0 / (74.0 * 73.0 * np.sqrt(k))).astype(np.float32)).to(DEV)
    offset = torch.from_numpy(rng.integers(-2000, 2000, n).astype(np.int32)).to(DEV)
    table = rng.permutation(256).astype(np.uint8).view(np.int8)   # a bijection: every code is told apart
    qp = P.make_qparams(z_r=-7)
    plain = torch.empty(m, n, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward(x, w, qp, mult, offset, None, None, P.CWAC_OUT_INT8, plain)
    full = torch.full((m, n + 16), 33, dtype=torch.int8, device=DEV)
    P.qlinear_cwac_forward_table(x, w, qp, mult, offset, _dev(table), full[:, :n],
                                 tuning=P.make_tuning(kernel=P.binding.CWAC_KERNEL_DIRECT_LDS) if force else None)
    torch.cuda.synchronize()
    codes = plain.cpu().numpy()
    assert np.unique(codes).size > 100                      # the codes spread over the range
    np.testing.assert_array_equal(full[:, :n].cpu().numpy(), table[codes.astype(int) + 128])
    assert (full[:, n:] == 33).all()
    if m >= 256 and n >= 256 and k % 128 == 0:
        # persistent workgroups that walk several tiles each (the table is staged once per workgroup)
        for wgs in (3, 7):
            again = torch.full((m, n + 16), 33, dtype=torch.int8, device=DEV)
            P.qlinear_cwac_forward_table(x, w, qp, mult, offset, _dev(table), again[:, :n],
                                         tuning=P.make_tuning(kernel=P.binding.CWAC_KERNEL_DIRECT_LDS,
                                                              shape=P.binding.CWAC_SHAPE_256_PERSIST,
                                                              persist_workgroups=wgs))
            torch.cuda.synchronize()
            assert torch.equal(again, full), wgs


def test_forward_with_code_table_argument_errors():
    x = torch.zeros(256, 64, dtype=torch.int8, device=DEV)
    w = torch.zeros(256, 64, dtype=torch.int8, device=DEV)
    mult = torch.ones(256, device=DEV)
    tab = torch.zeros(256, dtype=torch.int8, device=DEV)
    out = torch.empty(256, 264, dtype=torch.int8, device=DEV)
    with pytest.raises(P.CwacError):
        P.qlinear_cwac_forward_table(x, w[:250], P.make_qparams(), mult, None, tab, out[:, :250])   # n % 16
    with pytest.raises(P.CwacError):
        P.qlinear_cwac_forward_table(x, w, P.make_qparams(), mult, None, tab, out[:, 8:264])   # misaligned out
