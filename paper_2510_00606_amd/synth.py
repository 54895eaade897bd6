"""Seeded synthetic inputs: stand-ins for a training job's ZeRO state.

This module serves both the tests' CPU oracle and the GPU path and therefore holds none of the
method's arithmetic (no layout, no plan, no checksum): it only answers "what value does buffer
`tag`, array `arr`, position `i` hold?".  The generator is counter based, so any position can be
produced alone (for sampled checks of multi-gigabyte buffers) and on any torch device with the
same bits: integer hashing plus a table lookup and three single IEEE fp32 operations.

Value recipe (mixed-precision Adam state, Sec. 5.1):
  W (fp32 master), M, V (Adam moments): N(0, 0.02) by inverse-CDF sampling on a 2^16-bin
      quantile table with linear interpolation inside the bin (tails clipped at the outermost
      bin edge, about 4.3 sigma).  M and V are independent draws; V is not squared, only the bit
      patterns matter to a path that moves bytes.
  P (bf16 parameter): round-to-nearest-even of W at the same position.
"""
from __future__ import annotations

import functools

import numpy as np
import torch

ARRAYS = ("P", "W", "M", "V")
ELEM_SIZE = {"P": 2, "W": 4, "M": 4, "V": 4}
TORCH_DTYPE = {"P": torch.bfloat16, "W": torch.float32, "M": torch.float32, "V": torch.float32}
BYTES_PER_ELEMENT = 14
SIGMA = 0.02

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for the same bits."""
    x &= _M64
    return x - (1 << 64) if x >> 63 else x


def mix64_py(x: int) -> int:
    x = (x + _GOLDEN) & _M64
    x = ((x ^ (x >> 30)) * _C1) & _M64
    x = ((x ^ (x >> 27)) * _C2) & _M64
    return x ^ (x >> 31)


def stream_key(seed: int, tag: int, arr: str) -> int:
    """64-bit key of one buffer: `tag` names the buffer (e.g. old rank), `arr` the state array.
    P shares W's stream (it is W rounded)."""
    a = {"P": 1, "W": 1, "M": 2, "V": 3}[arr]
    return mix64_py(mix64_py(seed & _M64) ^ ((tag & 0xFFFFFFFF) << 8 | a))


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    x = x + _s64(_GOLDEN)
    x = (x ^ _lsr(x, 30)) * _s64(_C1)
    x = (x ^ _lsr(x, 27)) * _s64(_C2)
    return x ^ _lsr(x, 31)


@functools.lru_cache(maxsize=None)
def _edges_cpu() -> torch.Tensor:
    """2^16 + 1 bin edges of N(0, SIGMA): SIGMA * Phi^-1(i / 2^16), clipped tails.  Always
    computed on the CPU in float64 and then cast, so every device sees the same table."""
    from scipy.special import ndtri
    n = 1 << 16
    p = np.arange(n + 1, dtype=np.float64) / n
    p = np.clip(p, 0.5 / n, 1.0 - 0.5 / n)
    return torch.from_numpy((SIGMA * ndtri(p)).astype(np.float32))


_edges_dev: dict = {}


def _edges(device) -> torch.Tensor:
    key = str(device)
    if key not in _edges_dev:
        _edges_dev[key] = _edges_cpu().to(device)
    return _edges_dev[key]


def values_at(seed: int, tag: int, arr: str, idx: torch.Tensor) -> torch.Tensor:
    """Values of buffer (`tag`, `arr`) at int64 positions `idx` (any shape, any device)."""
    key = stream_key(seed, tag, arr)
    h = _mix64(idx * _s64(_GOLDEN) + _s64(key))
    e = _edges(idx.device)
    b = _lsr(h, 48)                                   # bin, 16 bits
    f = (_lsr(h, 24) & 0xFFFFFF).to(torch.float32) * (1.0 / (1 << 24))  # exact, in [0, 1)
    lo = e[b]
    w = lo + f * (e[b + 1] - lo)                      # three separately rounded fp32 ops
    if arr == "P":
        return w.to(torch.bfloat16)                   # round to nearest even
    return w


def fill(seed: int, tag: int, arr: str, start: int, count: int, device, batch: int = 1 << 26) -> torch.Tensor:
    """Positions [start, start+count) of buffer (`tag`, `arr`) as a new tensor on `device`."""
    out = torch.empty(count, dtype=TORCH_DTYPE[arr], device=device)
    for b0 in range(0, count, batch):
        n = min(batch, count - b0)
        idx = torch.arange(start + b0, start + b0 + n, dtype=torch.int64, device=device)
        out[b0:b0 + n] = values_at(seed, tag, arr, idx)
    return out


def to_numpy_bits(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor as unsigned integers of its element width (bf16 has no numpy dtype)."""
    t = t.detach().cpu().contiguous()
    if t.element_size() == 2:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.element_size() == 4:
        return t.view(torch.int32).numpy().view(np.uint32)
    if t.element_size() == 8:
        return t.view(torch.int64).numpy().view(np.uint64)
    return t.view(torch.uint8).numpy()
