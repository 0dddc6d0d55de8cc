"""Pins of the block-glue oracle (oracle/block_oracle.py) against things it does not call:
torch's fp64 layer_norm / gelu / softmax / scaled_dot_product_attention, closed forms, hand-worked
cases and invariants.  Each pin is chosen so that a plausible slip (unbiased variance, eps outside the
root, a transposed operand, a missing 1/sqrt(d), the tanh form of GELU, half-away-from-zero rounding,
a wrong head layout) fails it."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import block_oracle as blk


def _rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ layer normalization
def test_layernorm_against_library():
    rng = _rng(1)
    x = rng.standard_normal((7, 48)) * 3 + 1.5
    g = rng.standard_normal(48)
    b = rng.standard_normal(48)
    ref = F.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), 1e-6).numpy()
    np.testing.assert_allclose(blk.layernorm(x, g, b, 1e-6), ref, rtol=1e-12, atol=1e-12)


def test_layernorm_hand_worked_row():
    # x = (1, 2, 3, 4): mean 2.5, biased variance 1.25 (the unbiased one would be 5/3)
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    y = blk.layernorm(x, np.ones(4), np.zeros(4), 0.0)
    np.testing.assert_allclose(y[0], (x[0] - 2.5) / math.sqrt(1.25), rtol=1e-15)
    # eps sits under the root: with eps = 1.25 the divisor is sqrt(2.5)
    y = blk.layernorm(x, np.ones(4), np.zeros(4), 1.25)
    np.testing.assert_allclose(y[0], (x[0] - 2.5) / math.sqrt(2.5), rtol=1e-15)
    # gamma scales, beta shifts, per channel
    y = blk.layernorm(x, np.array([1.0, 2.0, 3.0, 4.0]), np.array([0.5, 0.0, 0.0, -1.0]), 0.0)
    z = (x[0] - 2.5) / math.sqrt(1.25)
    np.testing.assert_allclose(y[0], z * [1, 2, 3, 4] + [0.5, 0, 0, -1.0], rtol=1e-15)


def test_layernorm_invariants():
    rng = _rng(2)
    x = rng.standard_normal((5, 64))
    y = blk.layernorm(x, np.ones(64), np.zeros(64), 0.0)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose((y * y).mean(axis=1), 1, rtol=1e-13)
    # shift and positive scale of a row leave the normalized row unchanged
    y2 = blk.layernorm(3.0 * x + 7.0, np.ones(64), np.zeros(64), 0.0)
    np.testing.assert_allclose(y2, y, atol=1e-12)
    # rows are independent
    y3 = blk.layernorm(x[2:3], np.ones(64), np.zeros(64), 0.0)
    np.testing.assert_allclose(y3[0], y[2], rtol=1e-15)


# ------------------------------------------------------------------ quantizer
def test_quantize_ties_to_even_and_clipping():
    # s = 0.5, z = 3: y / s + z = y * 2 + 3
    y = np.array([0.25, 0.75, -0.25, -0.75, 1.0, 100.0, -100.0, 61.9, 62.3, -65.4, -65.6])
    c, v = blk.quantize(y, 0.5, 3)
    np.testing.assert_array_equal(v, y * 2 + 3)
    #        3.5->4  4.5->4  2.5->2  1.5->2  5   clip  clip  126.8->127  127.6->127  -127.8->-128  -128.2->-128
    np.testing.assert_array_equal(c, [4, 4, 2, 2, 5, 127, -128, 127, 127, -128, -128])
    assert c.dtype == np.int8
    # narrower code range (low-bit codes in int8 containers)
    c, _ = blk.quantize(np.array([10.0, -10.0, 1.5]), 1.0, 0, qmin=-8, qmax=7)
    np.testing.assert_array_equal(c, [7, -8, 2])


def test_dequantize_inverts_quantize_within_half_step():
    rng = _rng(3)
    y = rng.uniform(-3, 3, 1000)
    s, z = 6.0 / 255, -1
    c, _ = blk.quantize(y, s, z)
    assert np.abs(blk.dequantize(c, s, z) - y).max() <= s / 2 + 1e-12
    np.testing.assert_array_equal(blk.dequantize(np.array([-1, 0, 4], dtype=np.int8), 0.25, -1), [0.0, 0.25, 1.25])


# ------------------------------------------------------------------ GELU and its table
def test_gelu_against_library_and_closed_forms():
    x = np.linspace(-6, 6, 241)
    ref = F.gelu(torch.from_numpy(x)).numpy()  # erf form by default
    np.testing.assert_allclose(blk.gelu(x), ref, rtol=1e-13, atol=1e-15)
    assert blk.gelu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(blk.gelu(x) - blk.gelu(-x), x, atol=1e-14)  # x Phi(x) + x Phi(-x) = x
    # Phi(1) = 0.841344746068543: the tanh approximation gives 0.84119...
    np.testing.assert_allclose(blk.gelu(np.array([1.0]))[0], 0.8413447460685429, rtol=1e-14)


def test_gelu_table():
    s_in, z_in, s_out, z_out = 0.05, -20, 0.02, -120
    tab, v = blk.gelu_table(s_in, z_in, s_out, z_out)
    assert tab.shape == (256,) and tab.dtype == np.int8
    # entry of code c sits at index c + 128; code z_in is the real number 0 -> GELU 0 -> code z_out
    assert tab[z_in + 128] == z_out
    for code in (-128, -50, -20, 0, 37, 110):
        x = s_in * (code - z_in)
        g = 0.5 * x * (1 + math.erf(x / math.sqrt(2)))
        want = min(127, max(-128, round(g / s_out + z_out)))  # no tie among these
        assert abs((g / s_out + z_out) % 1 - 0.5) > 1e-6
        assert tab[code + 128] == want
        np.testing.assert_allclose(v[code + 128], g / s_out + z_out, rtol=1e-14)
    # monotone where GELU is (x >= -0.75 covers the minimum at -0.7518)
    xs = s_in * (np.arange(-128, 128) - z_in)
    inc = xs >= -0.75
    assert (np.diff(tab[inc].astype(int)) >= 0).all()


# ------------------------------------------------------------------ attention
def test_softmax_rows_against_library():
    rng = _rng(4)
    l = rng.standard_normal((6, 33)) * 4
    np.testing.assert_allclose(blk.softmax_rows(l), torch.softmax(torch.from_numpy(l), dim=-1).numpy(),
                               rtol=1e-13)
    # large logits do not overflow
    p = blk.softmax_rows(np.array([[1000.0, 1000.0, 0.0]]))
    np.testing.assert_allclose(p, [[0.5, 0.5, 0.0]], atol=1e-300)


def test_attention_against_library():
    rng = _rng(5)
    t, d = 19, 8
    q, k, v = (rng.standard_normal((t, d)) for _ in range(3))
    ref = F.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(k)[None],
                                         torch.from_numpy(v)[None])[0].numpy()
    o, mag = blk.attention(q, k, v)
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-13)
    assert (mag >= np.abs(o) - 1e-14).all()


def test_attention_bias_against_library_and_as_mask():
    rng = _rng(9)
    t, d = 13, 8
    q, k, v = (rng.standard_normal((t, d)) for _ in range(3))
    bias = rng.standard_normal((t, t))
    ref = F.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(k)[None],
                                         torch.from_numpy(v)[None], attn_mask=torch.from_numpy(bias)[None])[0].numpy()
    o, _ = blk.attention(q, k, v, bias)
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-13)
    # a bias that is constant along the keys changes nothing; a very negative column removes that key
    o0, _ = blk.attention(q, k, v)
    o1, _ = blk.attention(q, k, v, np.tile(rng.standard_normal((t, 1)), (1, t)))
    np.testing.assert_allclose(o1, o0, rtol=1e-12, atol=1e-13)
    mask = np.zeros((t, t))
    mask[:, 4] = -1e4
    o2, _ = blk.attention(q, k, v, mask)
    keep = np.arange(t) != 4
    o3, _ = blk.attention(q, k[keep], v[keep])
    np.testing.assert_allclose(o2, o3, rtol=1e-12, atol=1e-13)
    # per-head biases in the code-level entry point
    heads = 2
    r = rng.integers(-128, 128, (t, 3 * heads * d)).astype(np.int8)
    bh = rng.standard_normal((heads, t, t))
    ob, _ = blk.attention_codes(r, 0.05, 2, 1, t, heads, bh)
    x = 0.05 * (r.astype(np.float64) - 2)
    for h in range(heads):
        sl = slice(h * d, (h + 1) * d)
        oh, _ = blk.attention(x[:, sl], x[:, heads * d:][:, sl], x[:, 2 * heads * d:][:, sl], bh[h])
        np.testing.assert_allclose(ob[:, sl], oh, rtol=1e-13)


def test_attention_closed_forms():
    rng = _rng(6)
    t, d = 11, 4
    q = rng.standard_normal((t, d))
    # all keys equal: uniform weights, the output is the mean value row
    k = np.tile(rng.standard_normal((1, d)), (t, 1))
    v = rng.standard_normal((t, d))
    o, _ = blk.attention(q, k, v)
    np.testing.assert_allclose(o, np.tile(v.mean(axis=0), (t, 1)), rtol=1e-13)
    # one key and one value: the output is that value
    o, _ = blk.attention(q, k[:1], v[:1])
    np.testing.assert_allclose(o, np.tile(v[:1], (t, 1)), rtol=1e-15)
    # two keys, d = 4, q.k0 - q.k1 = 2 ln 3 * sqrt(d) / sqrt(d): weights 0.9 / 0.1 exactly when the
    # scaled logit difference is ln 9
    q1 = np.array([[math.log(9.0) * 2.0, 0, 0, 0]])     # / sqrt(4) -> ln 9 on key 0
    k2 = np.array([[1.0, 0, 0, 0], [0.0, 0, 0, 0]])
    v2 = np.array([[10.0, 0, 0, 0], [0.0, 10.0, 0, 0]])
    o, _ = blk.attention(q1, k2, v2)
    np.testing.assert_allclose(o[0], [9.0, 1.0, 0, 0], rtol=1e-13)


def test_attention_codes_head_layout():
    """Row = (q | k | v), head h in columns [h d, (h + 1) d) of each third; batches do not mix."""
    rng = _rng(7)
    batch, tokens, heads, d = 2, 5, 3, 4
    c = heads * d
    r = rng.integers(-128, 128, (batch * tokens, 3 * c)).astype(np.int8)
    s, z = 0.03, 5
    o, mag = blk.attention_codes(r, s, z, batch, tokens, heads)
    assert o.shape == (batch * tokens, c)
    x = torch.from_numpy(s * (r.astype(np.float64) - z)).reshape(batch, tokens, 3, heads, d)
    qh, kh, vh = (x[:, :, i].permute(0, 2, 1, 3) for i in range(3))          # [B, H, T, d]
    ref = F.scaled_dot_product_attention(qh, kh, vh).permute(0, 2, 1, 3).reshape(batch * tokens, c).numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-11, atol=1e-12)
    # changing batch 1 leaves batch 0 alone; changing head 2's values changes only head 2's columns
    r2 = r.copy()
    r2[tokens:, :] = 0
    o2, _ = blk.attention_codes(r2, s, z, batch, tokens, heads)
    np.testing.assert_array_equal(o2[:tokens], o[:tokens])
    r3 = r.copy()
    r3[:, 2 * c + 2 * d:2 * c + 3 * d] = 7
    o3, _ = blk.attention_codes(r3, s, z, batch, tokens, heads)
    np.testing.assert_array_equal(o3[:, :2 * d], o[:, :2 * d])
    np.testing.assert_allclose(o3[:, 2 * d:], s * (7 - z), rtol=1e-13)


# ------------------------------------------------------------------ residual stream
def test_residual_rounds_once_to_binary16():
    h = np.array([[1.0, 2048.0, -0.5, 1.0]], dtype=np.float16)
    codes = np.array([[3, 1, -4, 0]], dtype=np.int8)
    s, z = 2.0 ** -12, -1
    out, t = blk.residual(h, codes, s, z)
    # deq = 2^-12 * (code + 1).  1 + 4 * 2^-12 = 1 + 2^-10 is representable; 2048 + 2^-11 rounds back to 2048;
    # -0.5 - 3 * 2^-12 sits in [0.5, 1), spacing 2^-11: 1.5 spacings below -0.5, a tie, goes to the even
    # neighbour -0.5 - 2^-10; 1 + 2^-12 is a quarter of the spacing 2^-10 above 1 and rounds to 1
    np.testing.assert_array_equal(t, [[1 + 2.0 ** -10, 2048 + 2.0 ** -11, -0.5 - 3 * 2.0 ** -12, 1 + 2.0 ** -12]])
    np.testing.assert_array_equal(out.astype(np.float64),
                                  [[1 + 2.0 ** -10, 2048.0, -0.5 - 2.0 ** -10, 1.0]])
    assert out.dtype == np.float16
