"""Seeded, counter-based synthetic data: the only module both the HIP path's tests
and the CPU oracle's tests draw inputs from.  It holds no arithmetic of the
capture method itself (no gathers, no downcasts, no record layout).

Every value is a pure function of (seed, element index), built from integer
operations and one table lookup only, so the same bytes come out on the CPU and
on the GPU whatever the library versions of log/cos are:

    u   = splitmix64(seed, index) >> 48               (16 uniform bits)
    x   = TABLE[u]                                    (bf16)
    TABLE[k] = bf16_rne( Phi^-1((k + 0.5) / 65536) )  (standard-normal quantiles)

so activations are ~N(0,1) quantised to 65,536 equiprobable levels, which is
finer than bf16's own resolution around zero matters for a data-oblivious copy
path.  The table is always computed on the host (scipy's inverse normal CDF,
float64) and moved to the device as data.
"""
from __future__ import annotations

import functools

import numpy as np
import torch

BASE_SEED = 20260511

_GOLDEN = 0x9E3779B97F4A7C15
_MIX1 = 0xBF58476D1CE4E5B9
_MIX2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Two's-complement reinterpretation of a u64 constant as a Python int that
    fits torch.int64."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def splitmix64_scalar(seed: int, index: int) -> int:
    """Reference scalar form (Python ints) used to pin the vector forms."""
    z = (seed + (index + 1) * _GOLDEN) & _MASK64
    z = ((z ^ (z >> 30)) * _MIX1) & _MASK64
    z = ((z ^ (z >> 27)) * _MIX2) & _MASK64
    return z ^ (z >> 31)


def splitmix64_np(seed: int, index: np.ndarray) -> np.ndarray:
    idx = index.astype(np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _MASK64) + (idx + np.uint64(1)) * np.uint64(_GOLDEN)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_MIX1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_MIX2)
        return z ^ (z >> np.uint64(31))


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right on int64 (torch's >> is arithmetic)."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def splitmix64_torch(seed: int, index: torch.Tensor) -> torch.Tensor:
    """Same generator on int64 tensors (wrapping arithmetic), any device.
    Returns the 64 output bits reinterpreted as int64."""
    z = (index + 1) * _s64(_GOLDEN) + _s64(seed)
    z = (z ^ _lsr(z, 30)) * _s64(_MIX1)
    z = (z ^ _lsr(z, 27)) * _s64(_MIX2)
    return z ^ _lsr(z, 31)


@functools.lru_cache(maxsize=1)
def normal_table_u16() -> np.ndarray:
    """bf16 bit patterns of the 65,536 standard-normal quantile mid-points."""
    from scipy.special import ndtri

    q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    t = torch.from_numpy(q.astype(np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().astype(np.uint16)


@functools.lru_cache(maxsize=4)
def _normal_table_torch(device: str) -> torch.Tensor:
    t = torch.from_numpy(normal_table_u16().astype(np.int16)).view(torch.bfloat16)
    return t.to(device)


def sub_seed(*parts: int) -> int:
    """Derive a stream seed from BASE_SEED and small integer tags (config,
    point, pool slot ...)."""
    s = BASE_SEED
    for p in parts:
        s = splitmix64_scalar(s, int(p))
    return s


def randn_bf16(seed: int, n: int, device: str | torch.device = "cpu",
               chunk: int = 1 << 25, out: torch.Tensor | None = None) -> torch.Tensor:
    """n bf16 values ~N(0,1); element i depends on (seed, i) only."""
    device = torch.device(device)
    table = _normal_table_torch(str(device))
    if out is None:
        out = torch.empty(n, dtype=torch.bfloat16, device=device)
    assert out.numel() == n and out.dtype == torch.bfloat16 and out.is_contiguous()
    flat = out.view(-1)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        u = _lsr(splitmix64_torch(seed, idx), 48)
        flat[lo:hi] = table[u]
    return out


def randn_bf16_np(seed: int, n: int, start: int = 0) -> np.ndarray:
    """numpy route to the same bits (uint16 bf16 patterns) for elements
    [start, start+n)."""
    idx = np.arange(start, start + n, dtype=np.uint64)
    u = (splitmix64_np(seed, idx) >> np.uint64(48)).astype(np.int64)
    return normal_table_u16()[u]


def randint(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform in [lo, hi] (inclusive), host side."""
    r = splitmix64_np(seed, np.arange(n, dtype=np.uint64))
    return (lo + (r % np.uint64(hi - lo + 1)).astype(np.int64)).astype(np.int64)


def permutation(seed: int, n: int) -> np.ndarray:
    """Seeded permutation of 0..n-1 (argsort of the generator's outputs; ties
    are impossible to matter because argsort is stable)."""
    r = splitmix64_np(seed, np.arange(n, dtype=np.uint64))
    return np.argsort(r, kind="stable").astype(np.int64)
