"""Seeded synthetic inputs shared by the tests and the benchmark.

This module holds no arithmetic of the method: it only fills tensors.  The paper's own
workloads are random matrices (Section 4.3.1 builds A, B and C with ``rand``), so synthetic
inputs are the paper's workloads; entries here are i.i.d. uniform in [-1, 1).

The generator is counter-based: element ``i`` of stream ``s`` under seed ``q`` depends only on
(q, s, i), so any device (CPU or GPU) and any chunking produce bit-identical tensors.  All
integer steps are done in int64 with explicit 32-bit masks, which torch evaluates identically
on every backend.
"""
from __future__ import annotations

from typing import Tuple

import torch

DEFAULT_SEED = 200912263
_M32 = 0xFFFFFFFF
_CHUNK = 1 << 24


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """An avalanche permutation of 32-bit words (multiply / xor-shift rounds), on int64 storage."""
    x = ((x ^ (x >> 16)) * 0x7FEB352D) & _M32
    x = ((x ^ (x >> 15)) * 0x846CA68B) & _M32
    return x ^ (x >> 16)


def _mix32_int(x: int) -> int:
    x &= _M32
    x = ((x ^ (x >> 16)) * 0x7FEB352D) & _M32
    x = ((x ^ (x >> 15)) * 0x846CA68B) & _M32
    return x ^ (x >> 16)


def hash_u32(start: int, count: int, seed: int, stream: int, device) -> torch.Tensor:
    """32-bit hash of the counters start .. start+count-1 (int64 tensor holding values < 2**32)."""
    key = _mix32_int(seed * 0x9E3779B1 + stream * 0x85EBCA77 + 0x165667B1)
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    lo = idx & _M32
    hi = (idx >> 32) & _M32
    return _mix32(_mix32(lo ^ key) + _mix32(hi + 0x27D4EB2F) & _M32)


def _fill(numel: int, seed: int, stream: int, device, dtype, fn) -> torch.Tensor:
    out = torch.empty(numel, dtype=dtype, device=device)
    for s in range(0, numel, _CHUNK):
        n = min(_CHUNK, numel - s)
        out[s:s + n] = fn(hash_u32(s, n, seed, stream, device)).to(dtype)
    return out


def uniform_pm1(numel: int, stream: int, seed: int = DEFAULT_SEED, device="cpu",
                dtype=torch.float16) -> torch.Tensor:
    """Flat tensor of i.i.d. uniform values on the grid k / 2**23 - 1, k < 2**24, i.e. in [-1, 1);
    formed exactly in float32 and then rounded to nearest-even into ``dtype``."""
    return _fill(numel, seed, stream, device, dtype,
                 lambda h: (h >> 8).to(torch.float32) * (1.0 / 8388608.0) - 1.0)


def small_ints(numel: int, stream: int, seed: int = DEFAULT_SEED, device="cpu", dtype=torch.float16,
               lo: int = -8, hi: int = 8) -> torch.Tensor:
    """Flat tensor of integers in [lo, hi] (inclusive).  With |value| <= 8 every product and every
    partial sum of a K <= 2**18 dot product is an integer below 2**24, so FP32 accumulation is
    exact in any order: the result of the method is then unique and comparisons are bit-exact."""
    span = hi - lo + 1
    return _fill(numel, seed, stream, device, dtype, lambda h: ((h >> 4) % span + lo).to(torch.float32))


def stream_id(config: int, tensor: str) -> int:
    """A distinct stream number per (config, tensor name)."""
    return config * 64 + {"A": 0, "B": 1, "C": 2, "bias": 3, "A_im": 4, "B_im": 5, "C_im": 6, "d": 7}[tensor]


def col_major_strides(extents: Tuple[int, ...]) -> Tuple[int, ...]:
    """Dense strides with the first listed mode fastest ("column-major in listed mode order")."""
    st, s = [], 1
    for e in extents:
        st.append(s)
        s *= e
    return tuple(st)
