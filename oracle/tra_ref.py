"""tra_ref: the tensor-relational algebra written out literally on the CPU.  TEST INFRASTRUCTURE ONLY.

Follows Section 4 of the paper: a tensor relation is a map key -> sub-tensor
fixed by a bound vector b and a partitioning vector d (4.1); join applies a
kernel K to every pair of sub-tensors whose keys agree on shared labels and
names the result with the natural-join key; aggregation groups by the labels
that survive and reduces each group with (+); repartition re-slices (4.2).  An
EinSum with partitioning vector d is then join followed by aggregation (4.3),
where K is the same EinSum restricted to one pair of blocks.

Readings taken where the text is inconsistent:
  * d[i] is the NUMBER of slices along dimension i (Section 6), each of extent
    e = b/d; element j lives in block j div e at position j mod e.  This is the
    reading under which the d = [2,2] example of 4.1 and the index arithmetic
    i*50 + i' of 4.3 are consistent.
  * aggregation groups by the labels NOT in l_agg and its output key is the
    key restricted to those labels (the defining equation of 4.3), not the
    reverse as one sentence of 4.2 has it.
  * tuples are listed in row-major order of the key over the unique labels
    l_X (.) l_Y (first appearance order, last label fastest); the paper leaves
    the order open and any order is correct.

Parity unpinned: nothing here; every function is pinned by printed values of
the paper or by the decomposition invariant (see tests/test_oracle_*.py).
"""
from __future__ import annotations

import itertools
import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .einsum_ref import einsum_ref, split_spec

Key = Tuple[int, ...]


# ---------------------------------------------------------------------------- label algebra
def project(b: Sequence[int], l1: Sequence[str], l2: Sequence[str]) -> List[int]:
    """b[l1; l2]: entry i is b[j] where l1[i] == l2[j] (first such j)."""
    l2 = list(l2)
    return [b[l2.index(l)] for l in l1]


def concat_unique(lX: Sequence[str], lY: Sequence[str]) -> List[str]:
    """l_X (.) l_Y: concatenation with duplicate labels removed (natural-join schema)."""
    out: List[str] = []
    for l in list(lX) + list(lY):
        if l not in out:
            out.append(l)
    return out


def agg_labels(lX, lY, lZ) -> List[str]:
    """Labels of the inputs that do not occur in the output, in schema order."""
    return [l for l in concat_unique(lX, lY or []) if l not in lZ]


def index_set(b: Sequence[int]):
    """I(b) in row-major order."""
    return itertools.product(*[range(int(n)) for n in b])


def check_copartition(lXY: Sequence[str], d: Sequence[int]) -> None:
    """Entries of d that belong to the same label must be equal."""
    seen: Dict[str, int] = {}
    for l, v in zip(lXY, d):
        if seen.setdefault(l, v) != v:
            raise ValueError(f"label {l} partitioned {seen[l]} and {v} ways")


def join_count(lX, lY, d_full: Sequence[int]) -> int:
    """N(l_X, l_Y, d) = prod d[l_X (.) l_Y; l_XY] with d given over the concatenation l_XY."""
    lXY = list(lX) + list(lY)
    check_copartition(lXY, d_full)
    return math.prod(project(d_full, concat_unique(lX, lY), lXY))


def count_partitionings(N: int, D: int) -> int:
    """Ways to place N doublings into D label buckets."""
    return math.factorial(N + D - 1) // (math.factorial(N) * math.factorial(D - 1))


def viable(lX, lY, p: int) -> List[List[int]]:
    """All power-of-two partitioning vectors (over l_XY, co-partitioned) with exactly p join results."""
    uniq = concat_unique(lX, lY or [])
    lXY = list(lX) + list(lY or [])
    N = int(round(math.log2(p)))
    if 2 ** N != p:
        raise ValueError("p must be a power of two")
    out = []
    for combo in itertools.product(range(N + 1), repeat=len(uniq)):
        if sum(combo) == N:
            per = {l: 2 ** e for l, e in zip(uniq, combo)}
            out.append([per[l] for l in lXY])
    return out


# ---------------------------------------------------------------------------- tensor relations
class Relation:
    """key -> dense sub-tensor, with bound b and partitioning d (Section 4.1)."""

    def __init__(self, b: Sequence[int], d: Sequence[int], blocks: Dict[Key, np.ndarray], dtype: str):
        self.b = [int(x) for x in b]
        self.d = [int(x) for x in d]
        self.blocks = blocks
        self.dtype = dtype

    def extent(self) -> List[int]:
        return [bb // dd for bb, dd in zip(self.b, self.d)]


def partition(T: np.ndarray, d: Sequence[int], dtype: str = "f64") -> Relation:
    """Slice tensor T d[i] ways along dimension i into keyed sub-tensors."""
    b = list(T.shape)
    if len(d) != len(b):
        raise ValueError("d and b differ in length")
    for bb, dd in zip(b, d):
        if dd < 1 or bb % dd:
            raise ValueError(f"{dd} does not divide {bb}")
    e = [bb // dd for bb, dd in zip(b, d)]
    blocks = {}
    for key in index_set(d):
        sl = tuple(slice(k * ee, (k + 1) * ee) for k, ee in zip(key, e))
        blocks[key] = np.array(T[sl], copy=True)
    return Relation(b, d, blocks, dtype)


def assemble(R: Relation) -> np.ndarray:
    """The tensor equivalent to R: element j is block (j div e) at (j mod e)."""
    e = R.extent()
    first = next(iter(R.blocks.values()))
    out = np.empty(R.b, dtype=first.dtype)
    for j in index_set(R.b):
        key = tuple(jj // ee for jj, ee in zip(j, e))
        pos = tuple(jj % ee for jj, ee in zip(j, e))
        out[j] = R.blocks[key][pos]
    return out


def assemble_fast(R: Relation) -> np.ndarray:
    """Same tensor as assemble(), block copies instead of an element loop (for larger cases)."""
    e = R.extent()
    first = next(iter(R.blocks.values()))
    out = np.empty(R.b, dtype=first.dtype)
    for key, blk in R.blocks.items():
        sl = tuple(slice(k * ee, (k + 1) * ee) for k, ee in zip(key, e))
        out[sl] = blk
    return out


def repartition(R: Relation, d_new: Sequence[int]) -> Relation:
    """Pi_d: the relation with partitioning d_new equivalent to the same tensor."""
    return partition(assemble_fast(R), d_new, R.dtype)


def block_descriptor(b: Sequence[int], d: Sequence[int], key: Sequence[int], strides: Optional[Sequence[int]] = None):
    """(element offset, block bound, strides) of block `key` inside the dense row-major tensor."""
    b = [int(x) for x in b]
    if strides is None:
        strides, acc = [0] * len(b), 1
        for i in range(len(b) - 1, -1, -1):
            strides[i] = acc
            acc *= b[i]
    e = [bb // dd for bb, dd in zip(b, d)]
    off = sum(k * ee * s for k, ee, s in zip(key, e, strides))
    return off, e, list(strides)


# ---------------------------------------------------------------------------- TRA operators
def join(Xr: Relation, Yr: Relation, lX, lY, K):
    """All (key over l_X (.) l_Y, K(x, y)) for pairs whose keys agree on shared labels."""
    uniq = concat_unique(lX, lY)
    out = []
    for kx, xt in Xr.blocks.items():
        for ky, yt in Yr.blocks.items():
            if all(kx[i] == ky[j] for i, a in enumerate(lX) for j, c in enumerate(lY) if a == c):
                val = {}
                for l, k in zip(lX, kx):
                    val[l] = k
                for l, k in zip(lY, ky):
                    val[l] = k
                key = tuple(val[l] for l in uniq)
                out.append((key, kx, ky, K(xt, yt)))
    out.sort(key=lambda t: t[0])     # contract order: row-major over the schema key
    return uniq, out


def aggregate(temp, schema, l_agg, lZ, d_per_label: Dict[str, int], oplus: str):
    """Group by the labels not in l_agg; reduce each group in ascending aggIdx order."""
    groups: Dict[Key, List[Tuple[int, np.ndarray]]] = {}
    d_agg = [d_per_label[l] for l in schema if l in l_agg]
    for key, _kx, _ky, tensor in temp:
        val = dict(zip(schema, key))
        kz = tuple(val[l] for l in lZ)
        ka = [val[l] for l in schema if l in l_agg]
        agg_idx = 0
        for k, dd in zip(ka, d_agg):
            agg_idx = agg_idx * dd + k
        groups.setdefault(kz, []).append((agg_idx, tensor))
    out = {}
    for kz, members in groups.items():
        members.sort(key=lambda t: t[0])
        acc = members[0][1].copy()
        for _, t in members[1:]:
            acc = np.maximum(acc, t) if oplus == "max" else acc + t
        out[kz] = acc
    return out


def tuple_table(spec: str, d_unique: Sequence[int]):
    """The join's tuple table for partitioning d (per unique label), without touching data.

    Returns dict with: schema (unique labels), N, n_agg, d_X, d_Y, d_Z and per tuple
    key (over schema), keyX, keyY, keyZ, aggIdx, group (row-major rank of keyZ in I(d_Z)).
    """
    lX, lY, lZ = split_spec(spec)
    schema = concat_unique(lX, lY or [])
    if len(d_unique) != len(schema):
        raise ValueError("d must have one entry per unique label")
    dmap = dict(zip(schema, [int(x) for x in d_unique]))
    l_agg = [l for l in schema if l not in lZ]
    d_X = [dmap[l] for l in lX]
    d_Y = [dmap[l] for l in (lY or [])]
    d_Z = [dmap[l] for l in lZ]
    d_agg = [dmap[l] for l in l_agg]
    rows = []
    # literal join over key sets (a unary EinSum has a one-key right side)
    for kx in index_set(d_X):
        for ky in (index_set(d_Y) if lY else [()]):
            if all(kx[i] == ky[j] for i, a in enumerate(lX) for j, c in enumerate(lY or []) if a == c):
                val = dict(zip(lX, kx))
                val.update(dict(zip(lY or [], ky)))
                key = tuple(val[l] for l in schema)
                kz = tuple(val[l] for l in lZ)
                agg_idx = 0
                for l, dd in zip(l_agg, d_agg):
                    agg_idx = agg_idx * dd + val[l]
                group = 0
                for k, dd in zip(kz, d_Z):
                    group = group * dd + k
                rows.append(dict(key=key, keyX=tuple(kx), keyY=tuple(ky), keyZ=kz, aggIdx=agg_idx, group=group))
    rows.sort(key=lambda r: r["key"])
    return dict(schema=schema, N=len(rows), n_agg=math.prod(d_agg), d_X=d_X, d_Y=d_Y, d_Z=d_Z, rows=rows)


def tra_einsum(spec: str, X: np.ndarray, Y: Optional[np.ndarray], d_unique: Sequence[int], *,
               otimes: str = "mul", oplus: str = "sum", alpha: float = 1.0, out_dtype: str = "f64",
               x_dtype: Optional[str] = None, y_dtype: Optional[str] = None):
    """EinSum as join + aggregation over tensor relations (Section 4.3).

    Returns (dense Z as float64 rounded to out_dtype, number of kernel calls).
    The kernel K is einsum_ref on one pair of blocks with no rounding; partial
    blocks are reduced in double in ascending aggIdx order; one rounding at the end.
    """
    lX, lY, lZ = split_spec(spec)
    schema = concat_unique(lX, lY or [])
    dmap = dict(zip(schema, [int(x) for x in d_unique]))
    bmap = dict(zip(lX, X.shape))
    if lY:
        bmap.update(dict(zip(lY, Y.shape)))
    l_agg = [l for l in schema if l not in lZ]
    Xr = partition(X, [dmap[l] for l in lX])
    if lY:
        Yr = partition(Y, [dmap[l] for l in lY])
    else:
        Yr = Relation([], [], {(): None}, "f64")

    def K(xt, yt):
        return einsum_ref(spec, xt, yt, otimes=otimes, oplus=oplus, alpha=alpha, out_dtype="f64",
                          x_dtype=x_dtype, y_dtype=y_dtype)

    _, temp = join(Xr, Yr, lX, lY or [], K)
    res = aggregate(temp, schema, l_agg, lZ, dmap, oplus)
    Zr = Relation([bmap[l] for l in lZ], [dmap[l] for l in lZ], res, "f64")
    Z = assemble_fast(Zr) if lZ else np.asarray(res[()], dtype=np.float64).reshape(())
    if out_dtype == "f32":
        Z = Z.astype(np.float32).astype(np.float64)
    elif out_dtype == "bf16":
        from .einsum_ref import round_bf16
        Z = np.vectorize(round_bf16, otypes=[np.float64])(Z)
    return Z, len(temp)
