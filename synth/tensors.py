"""Counter-based, integer-only pseudo-normal generator.

value(seed, stream, i) depends only on its three integer arguments, so any
subset of elements can be produced on its own -- the whole buffer on the
GPU for the HIP path, a sample of indices on the CPU for the oracle -- and
the two agree bit for bit.  Everything up to the final int->float convert
and one fp32 multiply is integer arithmetic on values below 2**63 (no
wrap-around), written with torch ops that exist for both devices.

The variate is the centred sum of eight 16-bit uniforms (Irwin-Hall, n=8):
mean 0, excess kurtosis -0.15, support +-4.9 sigma.  It stands in for the
N(0, sigma^2) deltas and initial weights of the workload descriptions.
"""
from __future__ import annotations

import math
from typing import Union

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_MUL_A = 0x7FEB352D      # both multipliers are < 2**31, so x * mul < 2**63 for x < 2**32
_MUL_B = 0x31848BAB
# standard deviation of the sum of eight independent uniforms on {0..65535}
_SUM_STD = math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0)
_SUM_MEAN = 4 * 65535


def _mix32_int(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * _MUL_A) & _M32
    x ^= x >> 15
    x = (x * _MUL_B) & _M32
    x ^= x >> 14
    return x


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """Same mixer on an int64 tensor holding values in [0, 2**32)."""
    x = x ^ (x >> 16)
    x = (x * _MUL_A) & _M32
    x = x ^ (x >> 15)
    x = (x * _MUL_B) & _M32
    x = x ^ (x >> 14)
    return x


def _keys(seed: int, stream: int):
    base = _mix32_int(seed * 0x9E3779B1 + 0x1234567) ^ _mix32_int(stream * 0x85EBCA6B + 0x7654321)
    ka = [_mix32_int(base + 0x632BE5AB * (j + 1)) for j in range(4)]
    kb = [_mix32_int(base ^ (0x2545F491 * (j + 5))) for j in range(4)]
    return ka, kb


def _centred_sum(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """Integer variate in [-262140, 262140] for each element index (int64 tensor, values < 2**32)."""
    ka, kb = _keys(seed, stream)
    total = torch.zeros_like(idx)
    for j in range(4):
        h = _mix32(idx ^ ka[j])
        h = _mix32((h + kb[j]) & _M32)
        total = total + (h & 0xFFFF) + (h >> 16)
    return total - _SUM_MEAN


def scale_f32(sigma: float) -> np.float32:
    """The single fp32 factor that turns the integer variate into a value of std sigma."""
    return np.float32(sigma / _SUM_STD)


def normal_at(seed: int, stream: int, idx: torch.Tensor,
              scale: Union[float, np.float32, torch.Tensor]) -> torch.Tensor:
    """fp32 pseudo-normal values at the given flat element indices.

    idx    int64 tensor of element indices (0 <= idx < 2**32), any shape/device
    scale  fp32 factor from scale_f32(sigma): a scalar, or a float32 tensor
           broadcastable to idx (per-element sigma)
    """
    if idx.dtype != torch.int64:
        raise TypeError("idx must be int64")
    c = _centred_sum(seed, stream, idx).to(torch.float32)      # exact: |c| < 2**19
    if isinstance(scale, torch.Tensor):
        s = scale.to(device=idx.device, dtype=torch.float32)
    else:
        s = torch.tensor(float(np.float32(scale)), dtype=torch.float32, device=idx.device)
    return c * s                                               # one correctly rounded fp32 multiply


def normal_flat(seed: int, stream: int, start: int, count: int, scale: Union[float, np.float32],
                device: Union[str, torch.device] = "cpu", out: torch.Tensor | None = None,
                chunk: int = 1 << 24) -> torch.Tensor:
    """Values for the contiguous index range [start, start+count), generated in chunks.

    If `out` is given (float32, bfloat16 or float16, `count` elements) it is filled in
    place; 16-bit output is the fp32 value rounded to nearest-even.
    """
    if out is None:
        out = torch.empty(count, dtype=torch.float32, device=device)
    assert out.numel() == count
    flat = out.view(-1)
    for lo in range(0, count, chunk):
        hi = min(count, lo + chunk)
        idx = torch.arange(start + lo, start + hi, dtype=torch.int64, device=flat.device)
        flat[lo:hi] = normal_at(seed, stream, idx, scale).to(flat.dtype)
    return out


def to_bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """Round an fp32 tensor to bfloat16 (nearest-even) and return the raw 16-bit patterns as int16."""
    return x.to(torch.bfloat16).view(torch.int16)


def to_f16(x: torch.Tensor) -> torch.Tensor:
    """Round an fp32 tensor to IEEE half (nearest-even, subnormals kept)."""
    return x.to(torch.float16)
