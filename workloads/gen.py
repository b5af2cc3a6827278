"""Seeded, counter-based synthetic inputs, bit-identical on the host and on the GPU.

This module holds none of the method's arithmetic.  It only answers "what is the value of input
element number i of stream s under seed z", so that a 16 GiB cache can be filled on the device
chunk by chunk while a CPU check regenerates exactly the rows it wants to look at.

Recipe: a 32-bit integer mix of (seed, stream, index) picks one of 65536 equiprobable quantiles
of the standard normal (a table computed once on the host in float64 and rounded to float32);
the value is table[u] * sigma, rounded once to the requested dtype.  Integer mixing, a gather,
one IEEE float32 multiply and one round-to-nearest-even conversion give the same bits from
torch on the CPU and on the GPU.  The law is N(0, sigma^2) discretised to 2^16 levels, so it is
clipped at about +-4.3 sigma.
"""
from __future__ import annotations

import functools

import numpy as np
import torch

_M32 = 0xFFFFFFFF


@functools.lru_cache(maxsize=None)
def _quantile_table_cpu() -> torch.Tensor:
    from scipy.special import ndtri

    u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return torch.from_numpy(ndtri(u).astype(np.float32))


_table_cache: dict = {}


def _quantile_table(device) -> torch.Tensor:
    key = str(device)
    if key not in _table_cache:
        _table_cache[key] = _quantile_table_cpu().to(device)
    return _table_cache[key]


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """Avalanche a value in [0, 2^32) held in int64 (xor-shift / multiply rounds)."""
    x = x ^ (x >> 16)
    x = (x * 0x7FEB352D) & _M32
    x = x ^ (x >> 15)
    x = (x * 0x846CA68B) & _M32
    x = x ^ (x >> 16)
    return x


def uniform16(index: torch.Tensor, seed: int, stream: int) -> torch.Tensor:
    """16 pseudo-random bits per element of the int64 tensor `index` (values < 2^62)."""
    key = ((seed * 0x9E3779B1) ^ (stream * 0x85EBCA77) ^ 0x5BD1E995) & _M32
    hi = (index >> 32) & _M32
    lo = index & _M32
    h = _mix32(hi ^ key)
    h = _mix32(lo ^ h)
    return h & 0xFFFF


def normal(index: torch.Tensor, seed: int, stream: int, sigma: float, dtype: torch.dtype) -> torch.Tensor:
    """N(0, sigma^2)-like values for logical element numbers `index`, on index.device."""
    u = uniform16(index, seed, stream)
    x = _quantile_table(index.device)[u]
    if sigma != 1.0:
        x = x * torch.tensor(sigma, dtype=torch.float32, device=index.device)
    return x.to(dtype)


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a float32/bf16/fp16 tensor to a float64 numpy array."""
    return t.detach().cpu().to(torch.float64).numpy()


def to_bits(t: torch.Tensor) -> np.ndarray:
    """Raw storage words: uint16 for 16-bit formats, float32 (bit-comparable via view) otherwise."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy().view(np.uint32)
    raise TypeError(t.dtype)
