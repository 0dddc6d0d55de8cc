"""CPU oracle for the glue between the quantized linear layers of a Transformer block.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  It shares no code,
table or helper with the HIP sources.

The paper compensates every linear layer on its own precisely because the rest
of the block is non-linear (Sec. 3.2); it does not define that rest.  What is
written out here is the standard pre-norm Vision Transformer block with the
W8A8 linear layers of Sec. 3.4 in it (every linear layer consumes int8 codes and
requantizes its output to int8 codes, Eq. 10):

    x1 = Q(LN1(h))              r1 = qkv(x1)            int8 codes, (s, z)
    a  = Q(MHSA(deq(r1)))       r2 = proj(a)
    h1 = RN16(h + deq(r2))      x2 = Q(LN2(h1))         r3 = fc1(x2)
    g  = Q(GELU(deq(r3)))       r4 = fc2(g)
    h2 = RN16(h1 + deq(r4))

with Q(y) = clip(rne(y / s) + z, -128, 127) (Eq. 1, signed relabelling),
deq(c) = s * (c - z), LN the layer normalization over the channel axis (biased
variance), MHSA = softmax(Q K^T / sqrt(d)) V per head, GELU the erf form, and
the residual stream held in IEEE binary16.  Everything is evaluated in fp64 with
numpy; nothing is blocked, fused or reordered.  Every function returns the real
number BEFORE a rounding decision next to the decision itself, so that a test
can tell a wrong result from a tie that fp32 arithmetic may resolve either way.

Parity status: every function is pinned in tests/test_oracle_block.py against
library routines it does not call (torch's layer_norm, gelu, softmax and
scaled_dot_product_attention in fp64), closed forms and hand-worked cases.
"""
from __future__ import annotations

import math

import numpy as np


def layernorm(x, gamma, beta, eps):
    """y[m, c] = (x[m, c] - mean_m) / sqrt(var_m + eps) * gamma[c] + beta[c]; var = mean of the
    squared deviations (biased)."""
    x = np.asarray(x, dtype=np.float64)
    mean = x.sum(axis=1, keepdims=True) / x.shape[1]
    dev = x - mean
    var = (dev * dev).sum(axis=1, keepdims=True) / x.shape[1]
    y = dev / np.sqrt(var + float(eps))
    return y * np.asarray(gamma, dtype=np.float64)[None, :] + np.asarray(beta, dtype=np.float64)[None, :]


def quantize(y, s, z, qmin=-128, qmax=127):
    """Eq. 1 on signed codes -> (codes int8, v) with v = y / s + z the real number whose rounding
    to the nearest integer (ties to even), clipped, is the code."""
    v = np.asarray(y, dtype=np.float64) / float(s) + float(z)
    c = np.clip(np.rint(v), qmin, qmax)
    return c.astype(np.int8), v


def dequantize(codes, s, z):
    return float(s) * (np.asarray(codes).astype(np.float64) - float(z))


def gelu(x):
    """x * Phi(x) with the exact normal distribution function (erf form)."""
    x = np.asarray(x, dtype=np.float64)
    erf = np.vectorize(math.erf, otypes=[np.float64])
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def gelu_table(s_in, z_in, s_out, z_out, qmin=-128, qmax=127):
    """The 256-entry table code_in -> Q(GELU(deq(code_in))), indexed by code_in + 128
    -> (table int8 [256], v [256])."""
    codes = np.arange(-128, 128)
    return quantize(gelu(dequantize(codes, s_in, z_in)), s_out, z_out, qmin, qmax)


def softmax_rows(logits):
    m = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, bias=None):
    """softmax(q k^T / sqrt(d) + bias) v for one head; q, k, v [T, d], bias [T, T] or None -> (o [T, d],
    mag [T, d]) with mag = softmax(.) |v|, the scale of the rounding error of a lower-precision evaluation."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    logits = q @ k.T / math.sqrt(q.shape[1])
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=np.float64)
    p = softmax_rows(logits)
    return p @ v, p @ np.abs(v)


def attention_codes(r_qkv, s, z, batch, tokens, heads, bias=None):
    """Multi-head self-attention on the requantized output of the qkv layer.
    r_qkv: int8 codes [batch * tokens, 3 * C], row = (q | k | v), each C = heads * d wide with
    head h in columns [h * d, (h + 1) * d); bias [heads, tokens, tokens] (added to every image's logits) or
    None -> (o [batch * tokens, C], mag) in fp64."""
    r = np.asarray(r_qkv)
    c3 = r.shape[1]
    c = c3 // 3
    d = c // heads
    x = dequantize(r, s, z).reshape(batch, tokens, 3, heads, d)
    o = np.empty((batch, tokens, heads, d), dtype=np.float64)
    mag = np.empty_like(o)
    for b in range(batch):
        for h in range(heads):
            o[b, :, h, :], mag[b, :, h, :] = attention(x[b, :, 0, h, :], x[b, :, 1, h, :], x[b, :, 2, h, :],
                                                       None if bias is None else bias[h])
    return o.reshape(batch * tokens, c), mag.reshape(batch * tokens, c)


def residual(h16, codes, s, z):
    """h + deq(codes) -> (its nearest binary16 value, the fp64 sum)."""
    h16 = np.asarray(h16)
    assert h16.dtype == np.float16
    t = h16.astype(np.float64) + dequantize(codes, s, z)
    return t.astype(np.float16), t
