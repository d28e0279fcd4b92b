"""The same counter-based generator as prng.py, evaluated with torch integer ops on any device.

Used to fill multi-GiB inputs directly in HBM; element (seed, tensor_id, index) is bit-identical to the
numpy version (tests/test_inputs.py checks that), so the oracle can regenerate any sampled sub-range on
the host.  No arithmetic of the einsum method lives here.
"""
from __future__ import annotations

import math

import torch

_G = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_CHUNK = 1 << 26


def _s64(x: int) -> int:
    """Two's-complement view of a 64-bit constant (torch has no uint64 arithmetic)."""
    x &= 0xFFFFFFFFFFFFFFFF
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(z: torch.Tensor, n: int) -> torch.Tensor:
    """Logical shift right of int64 values."""
    return (z >> n) & ((1 << (64 - n)) - 1)


def hash_i64(seed: int, tensor_id: int, index: torch.Tensor) -> torch.Tensor:
    base = _s64((tensor_id + 1) * _G + (seed + 1) * _C1)
    z = index * _s64(_G) + base                     # wraps modulo 2^64
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def _fill(n: int, device, fn) -> torch.Tensor:
    out = torch.empty(n, dtype=torch.float32, device=device)
    for pos in range(0, n, _CHUNK):
        m = min(_CHUNK, n - pos)
        idx = torch.arange(pos, pos + m, dtype=torch.int64, device=device)
        out[pos:pos + m] = fn(idx)
    return out


def uniform_pm1(seed: int, tensor_id: int, n: int, device="cuda") -> torch.Tensor:
    def fn(idx):
        z = hash_i64(seed, tensor_id, idx)
        u = _lsr(z, 11).to(torch.float64) * (1.0 / 9007199254740992.0)
        return (2.0 * u - 1.0).to(torch.float32)
    return _fill(n, device, fn)


def normal(seed: int, tensor_id: int, n: int, std: float, device="cuda") -> torch.Tensor:
    def fn(idx):
        z = hash_i64(seed, tensor_id, idx)
        u1 = (_lsr(z, 32).to(torch.float64) + 1.0) * (1.0 / 4294967296.0)
        u2 = (z & 0xFFFFFFFF).to(torch.float64) * (1.0 / 4294967296.0)
        g = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)
        return (std * g).to(torch.float32)
    return _fill(n, device, fn)


def onehot(seed: int, tensor_id: int, rows: int, classes: int, device="cuda") -> torch.Tensor:
    z = hash_i64(seed, tensor_id, torch.arange(rows, dtype=torch.int64, device=device))
    cls = _lsr(z, 17) % classes
    out = torch.zeros((rows, classes), dtype=torch.float32, device=device)
    out[torch.arange(rows, device=device), cls] = 1.0
    return out


def make_tensor(recipe: dict, shape, dtype: str, seed: int, tensor_id: int, device="cuda") -> torch.Tensor:
    """Device tensor in its storage dtype ('f32' -> float32, 'bf16' -> bfloat16, round-to-nearest-even)."""
    shape = tuple(int(s) for s in shape)
    n = 1
    for s in shape:
        n *= s
    dist = recipe["dist"]
    if dist == "uniform":
        x = uniform_pm1(seed, tensor_id, n, device)
    elif dist == "normal":
        x = normal(seed, tensor_id, n, float(recipe["std"]), device)
    elif dist == "onehot":
        x = onehot(seed, tensor_id, shape[0], shape[1], device)
    elif dist == "causal_mask":
        x = torch.zeros(shape, dtype=torch.float32, device=device)
        x.masked_fill_(torch.triu(torch.ones(shape, dtype=torch.bool, device=device), diagonal=1), float("-inf"))
    elif dist == "ones":
        x = torch.ones(n, dtype=torch.float32, device=device)
    else:
        raise ValueError(f"unsupported dist {dist} for the device generator")
    x = x.reshape(shape)
    return x if dtype == "f32" else x.to(torch.bfloat16)
