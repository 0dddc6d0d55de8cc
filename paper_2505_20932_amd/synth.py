"""Seeded synthetic inputs for the five workloads (layer shapes and activation
statistics of ViT / Swin / LLM linears).

This module only draws random tensors.  It contains none of the method's
arithmetic (no quantizer, no GEMM, no fit): tests feed the very same arrays to
the CPU oracle and to the GPU library.

Generator: counter based.  Element pair ``j`` of stream ``(seed, stream)`` is
``splitmix64(seed, stream, j)`` -> two 24-bit uniforms -> Box-Muller.  It is
written with torch integer/float ops so that it runs on the host (tests) or on
the device (benchmark) from the same code; values depend only on
``(seed, stream, index)``, up to the device's log/sin/cos rounding.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

_GAMMA = -7046029254386353131          # 0x9E3779B97F4A7C15 as int64
_C1 = -4658895280553007687             # 0xBF58476D1CE4E5B9
_C2 = -7723592293110705685             # 0x94D049BB133111EB
_CHUNK = 1 << 24


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def _splitmix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _C1
    z = (z ^ _lsr(z, 27)) * _C2
    return z ^ _lsr(z, 31)


def _key(seed: int, stream: int) -> int:
    k = (seed * 0x632BE59BD9B4E019 + stream * 0x2545F4914F6CDD1D + 0x1234567) & ((1 << 64) - 1)
    return k - (1 << 64) if k >= (1 << 63) else k


def normal(seed: int, stream: int, count: int, device="cpu", start: int = 0) -> torch.Tensor:
    """Elements ``start .. start+count`` of the standard-normal stream
    ``(seed, stream)`` (fp32, 1-D)."""
    first = start // 2
    last = (start + count + 1) // 2
    out = torch.empty(2 * (last - first), dtype=torch.float32, device=device)
    key = _key(seed, stream)
    for p0 in range(first, last, _CHUNK):
        p1 = min(last, p0 + _CHUNK)
        idx = torch.arange(p0, p1, dtype=torch.int64, device=device)
        h = _splitmix(_splitmix(idx * _GAMMA + key))
        u1 = (((h >> 40) & 0xFFFFFF).to(torch.float32) + 1.0) * (1.0 / 16777216.0)
        u2 = ((h >> 8) & 0xFFFFFF).to(torch.float32) * (1.0 / 16777216.0)
        r = torch.sqrt(-2.0 * torch.log(u1))
        ang = (2.0 * math.pi) * u2
        seg = out[2 * (p0 - first):2 * (p1 - first)].view(-1, 2)
        seg[:, 0] = r * torch.cos(ang)
        seg[:, 1] = r * torch.sin(ang)
    off = start - 2 * first
    return out[off:off + count]


_M64 = (1 << 64) - 1


def _splitmix_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def uniform_ints(seed: int, stream: int, count: int, high: int) -> List[int]:
    """``count`` distinct integers in [0, high), host side (channel picks)."""
    picks: List[int] = []
    key = _key(seed, stream)
    j = 0
    while len(picks) < count:
        v = _splitmix_int(_splitmix_int(j * 0x9E3779B97F4A7C15 + key)) % high
        if v not in picks:
            picks.append(v)
        j += 1
    return picks


# ---------------------------------------------------------------------------
# workloads
# ---------------------------------------------------------------------------
@dataclass(frozen=True)
class Layer:
    name: str
    n: int          # output channels (C_out)
    k: int          # input channels (C_in)


@dataclass(frozen=True)
class Workload:
    cfg: int
    name: str
    m: int                      # token rows of the inference batch
    cal_rows: int               # calibration samples x tokens
    layers: Tuple[Layer, ...]
    per_token: bool = False     # per-token symmetric activation scales
    bias: bool = True
    outlier: str = "none"       # none | scale | student_t | lognormal
    outlier_frac: float = 0.0   # fraction of input channels (or a count if >= 1)
    outlier_gain: float = 1.0
    w_std: float = 0.02

    def seed(self, layer_index: int) -> int:
        return 0 if self.cfg == 1 else 1000 * self.cfg + layer_index


def _vit_block(i: int) -> Tuple[Layer, ...]:
    return (Layer(f"blk{i}.qkv", 2304, 768), Layer(f"blk{i}.proj", 768, 768),
            Layer(f"blk{i}.fc1", 3072, 768), Layer(f"blk{i}.fc2", 768, 3072))


WORKLOADS = {
    1: Workload(1, "deit_s_qkv", 197, 32 * 197, (Layer("qkv", 1152, 384),),
                outlier="scale", outlier_frac=4, outlier_gain=20.0),
    2: Workload(2, "vit_b16_fc1", 64 * 197, 256 * 197, (Layer("fc1", 3072, 768),),
                outlier="scale", outlier_frac=0.01, outlier_gain=30.0),
    3: Workload(3, "vit_b16_12blocks", 128 * 197, 512 * 197,
                tuple(l for i in range(12) for l in _vit_block(i)),
                outlier="student_t", outlier_frac=0.05),
    4: Workload(4, "swin_b_stage3", 128 * 196, 1024 * 196,
                (Layer("qkv", 1536, 512), Layer("fc1", 2048, 512), Layer("fc2", 512, 2048))),
    5: Workload(5, "llm_7b_decoder_layer", 8 * 2048, 128 * 2048,
                (Layer("qkv", 12288, 4096), Layer("o", 4096, 4096), Layer("up", 11008, 4096),
                 Layer("gate", 11008, 4096), Layer("down", 4096, 11008)),
                per_token=True, bias=False, outlier="lognormal", outlier_frac=0.002,
                outlier_gain=100.0),
}

# stream ids within one (workload, layer) seed
_S_PICK, _S_GAIN, _S_W, _S_B, _S_X, _S_XCAL, _S_T = 1, 2, 3, 4, 5, 6, 16


def _n_outlier(wl: Workload, k: int) -> int:
    if wl.outlier == "none":
        return 0
    if wl.outlier_frac >= 1:
        return int(wl.outlier_frac)
    return max(1, int(round(wl.outlier_frac * k)))


def activations(wl: Workload, layer_index: int, rows: int, calibration: bool = False,
                device="cpu", row0: int = 0) -> torch.Tensor:
    """fp32 layer input [rows, K]: N(0,1) with the workload's outlier channels.
    ``calibration`` selects the calibration stream; ``row0`` offsets into it so
    that a calibration set can be produced chunk by chunk."""
    k = wl.layers[layer_index].k
    seed = wl.seed(layer_index)
    stream = _S_XCAL if calibration else _S_X
    # whole rows are consumed in order, so chunk (row0, rows) is a slice of the stream
    x = normal(seed, stream, rows * k, device, start=row0 * k).view(rows, k).clone()
    n_out = _n_outlier(wl, k)
    if n_out == 0:
        return x
    chans = uniform_ints(seed, _S_PICK, n_out, k)
    ch = torch.tensor(chans, dtype=torch.int64, device=device)
    if wl.outlier == "scale":
        x[:, ch] *= wl.outlier_gain
    elif wl.outlier == "lognormal":
        g = normal(seed, _S_GAIN, n_out, device)
        x[:, ch] *= wl.outlier_gain * torch.exp(0.5 * g)
    elif wl.outlier == "student_t":
        # t(nu=3) = z / sqrt(chi2_3 / 3), chi2_3 from three more normals per element
        tstream = _S_T + (8 if calibration else 0)
        aux = normal(seed, tstream, rows * n_out * 3, device, start=row0 * n_out * 3)
        aux = aux.view(rows, n_out, 3)
        chi2 = (aux * aux).sum(dim=2)
        x[:, ch] = x[:, ch] / torch.sqrt(chi2 / 3.0)
    return x


def weights(wl: Workload, layer_index: int, device="cpu") -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """fp32 weight [N, K] ~ N(0, w_std^2) and bias [N] ~ N(0, w_std^2) (or None)."""
    ly = wl.layers[layer_index]
    seed = wl.seed(layer_index)
    w = normal(seed, _S_W, ly.n * ly.k, device).view(ly.n, ly.k) * wl.w_std
    b = normal(seed, _S_B, ly.n, device) * wl.w_std if wl.bias else None
    return w, b
