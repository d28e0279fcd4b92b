"""Counter-based input generator: value = f(seed, tensor_id, flat_index).

Every element is a pure function of three integers, so the oracle and the GPU
side see identical inputs without sharing generator state, and a sampled
sub-range of a huge tensor can be regenerated on its own.  Values are produced
in fp32 and then rounded to the storage dtype; both sides consume the rounded
values.
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_G = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_CHUNK = 1 << 22


def hash_u64(seed: int, tensor_id: int, index: np.ndarray) -> np.ndarray:
    """splitmix64-style finaliser over (seed, tensor_id, index); index is uint64."""
    with np.errstate(over="ignore"):
        base = np.uint64(((tensor_id + 1) * _G + (seed + 1) * _C1) & 0xFFFFFFFFFFFFFFFF)
        z = index.astype(np.uint64) * np.uint64(_G) + base
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_C1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_C2)
        z = z ^ (z >> np.uint64(31))
    return z


def _chunks(n: int, start: int = 0):
    pos = 0
    while pos < n:
        m = min(_CHUNK, n - pos)
        yield pos, np.arange(start + pos, start + pos + m, dtype=np.uint64)
        pos += m


def uniform_pm1(seed: int, tensor_id: int, n: int, start: int = 0) -> np.ndarray:
    """n fp32 values uniform in [-1, 1)."""
    out = np.empty(n, dtype=np.float32)
    for pos, idx in _chunks(n, start):
        z = hash_u64(seed, tensor_id, idx)
        u = (z >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        out[pos:pos + idx.size] = (2.0 * u - 1.0).astype(np.float32)
    return out


def normal(seed: int, tensor_id: int, n: int, std: float, start: int = 0) -> np.ndarray:
    """n fp32 values ~ N(0, std^2) by Box-Muller on the two 32-bit halves of one hash."""
    out = np.empty(n, dtype=np.float32)
    for pos, idx in _chunks(n, start):
        z = hash_u64(seed, tensor_id, idx)
        u1 = ((z >> np.uint64(32)).astype(np.float64) + 1.0) * (1.0 / 4294967296.0)
        u2 = (z & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[pos:pos + idx.size] = (std * g).astype(np.float32)
    return out


def small_ints(seed: int, tensor_id: int, n: int, lo: int = -2, hi: int = 2, start: int = 0) -> np.ndarray:
    """n fp32 values that are integers in [lo, hi]; sums of products stay exact in fp32."""
    out = np.empty(n, dtype=np.float32)
    span = np.uint64(hi - lo + 1)
    for pos, idx in _chunks(n, start):
        z = hash_u64(seed, tensor_id, idx)
        out[pos:pos + idx.size] = ((z >> np.uint64(20)) % span).astype(np.float32) + np.float32(lo)
    return out


def onehot(seed: int, tensor_id: int, rows: int, classes: int) -> np.ndarray:
    """[rows, classes] fp32 one-hot matrix; the hot class of each row is uniform over classes."""
    z = hash_u64(seed, tensor_id, np.arange(rows, dtype=np.uint64))
    cls = ((z >> np.uint64(17)) % np.uint64(classes)).astype(np.int64)
    out = np.zeros((rows, classes), dtype=np.float32)
    out[np.arange(rows), cls] = 1.0
    return out


def causal_mask(s: int, t: int) -> np.ndarray:
    """[s, t] fp32 additive mask: 0 where t <= s, -inf above the diagonal."""
    m = np.zeros((s, t), dtype=np.float32)
    m[np.triu_indices(s, k=1, m=t)] = -np.inf
    return m


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    inf_nan = (b & np.uint32(0x7F800000)) == np.uint32(0x7F800000)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    r = np.where(inf_nan, b >> np.uint32(16), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class HostTensor:
    """A dense row-major host tensor in its storage dtype.

    dtype 'f32': data is float32.  dtype 'bf16': data is uint16 bit patterns.
    """
    data: np.ndarray
    dtype: str

    @property
    def shape(self):
        return tuple(self.data.shape)

    def as_f32(self) -> np.ndarray:
        return self.data if self.dtype == "f32" else bf16_bits_to_f32(self.data).reshape(self.data.shape)

    def as_f64(self) -> np.ndarray:
        return self.as_f32().astype(np.float64)

    @staticmethod
    def from_f32(x: np.ndarray, dtype: str) -> "HostTensor":
        x = np.ascontiguousarray(x, dtype=np.float32)
        if dtype == "f32":
            return HostTensor(x, "f32")
        if dtype == "bf16":
            return HostTensor(f32_to_bf16_bits(x).reshape(x.shape), "bf16")
        raise ValueError(dtype)


def make_tensor(recipe: dict, shape, dtype: str, seed: int, tensor_id: int) -> HostTensor:
    """Materialise one input tensor from its recipe.

    recipe['dist'] is one of: 'uniform' (U[-1,1)), 'normal' (needs 'std'),
    'ints' (small integers lo..hi), 'onehot' (rank 2), 'causal_mask' (rank 2),
    'ones', 'identity' (rank 2), 'const' (needs 'value').
    """
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape)) if shape else 1
    dist = recipe["dist"]
    if dist == "uniform":
        x = uniform_pm1(seed, tensor_id, n)
    elif dist == "normal":
        x = normal(seed, tensor_id, n, float(recipe["std"]))
    elif dist == "ints":
        x = small_ints(seed, tensor_id, n, int(recipe.get("lo", -2)), int(recipe.get("hi", 2)))
    elif dist == "onehot":
        x = onehot(seed, tensor_id, shape[0], shape[1])
    elif dist == "causal_mask":
        x = causal_mask(shape[0], shape[1])
    elif dist == "ones":
        x = np.ones(n, dtype=np.float32)
    elif dist == "identity":
        x = np.eye(shape[0], shape[1], dtype=np.float32)
    elif dist == "const":
        x = np.full(n, float(recipe["value"]), dtype=np.float32)
    else:
        raise ValueError(f"unknown dist {dist}")
    return HostTensor.from_f32(np.asarray(x, dtype=np.float32).reshape(shape), dtype)
