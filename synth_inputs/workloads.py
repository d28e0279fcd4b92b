"""Plain-data descriptions of the einsum graphs used as workloads.

A workload is an EinGraph in the paper's sense (Section 5: one triple
(bound, EinSum, inputs) per vertex) plus named sets of partitioning vectors
(one per einsum vertex, Section 6).  Nothing here evaluates anything: the
oracle and the HIP library each translate these records on their own.

The five configurations mirror the paper's experiments with synthetic data:
matrix-chain arithmetic (Experiment 1), an FFNN training step on a wide
classifier (Experiment 2) and a LLaMA-like decoder block prefill
(Experiment 3).  Their datasets and weights are replaced by seeded random
tensors of the same shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

SEED_BASE = 241002682


@dataclass
class Vertex:
    name: str
    dtype: str                               # storage dtype of this vertex's tensor: 'f32' | 'bf16'
    bound: Optional[Tuple[int, ...]] = None  # graph inputs only
    recipe: Optional[dict] = None            # graph inputs only (see prng.make_tensor)
    spec: Optional[str] = None               # "ij,jk->ik" (binary) or "ij->i" (unary)
    otimes: str = "mul"                      # scalar join / map function
    oplus: str = "sum"                       # 'sum' | 'max' | 'none' (no aggregated label)
    alpha: float = 1.0                       # scalar parameter of otimes
    inputs: Tuple[str, ...] = ()

    @property
    def is_input(self) -> bool:
        return self.spec is None


@dataclass
class Workload:
    name: str
    seed: int
    vertices: List[Vertex]
    outputs: List[str]
    # partitionings[name][vertex_name] = {label: d}; labels not listed are unsplit.
    partitionings: Dict[str, Dict[str, Dict[str, int]]] = field(default_factory=dict)
    dims: Dict[str, int] = field(default_factory=dict)

    def vertex(self, name: str) -> Vertex:
        for v in self.vertices:
            if v.name == name:
                return v
        raise KeyError(name)

    def einsum_vertices(self) -> List[Vertex]:
        return [v for v in self.vertices if not v.is_input]

    def tensor_id(self, name: str) -> int:
        return [v.name for v in self.vertices].index(name)


def parse_spec(spec: str):
    """'ij,jk->ik' -> (['i','j'], ['j','k'], ['i','k']); unary has lY = None.  Pure string handling."""
    lhs, rhs = spec.split("->")
    ops = lhs.split(",")
    lX = list(ops[0])
    lY = list(ops[1]) if len(ops) > 1 else None
    return lX, lY, list(rhs)


def unique_labels(spec: str) -> List[str]:
    """Unique labels in first-appearance order over lX then lY (the natural-join schema)."""
    lX, lY, _ = parse_spec(spec)
    out: List[str] = []
    for l in lX + (lY or []):
        if l not in out:
            out.append(l)
    return out


def d_vector(spec: str, part: Dict[str, int]) -> List[int]:
    """Partitioning vector per unique label for one vertex from a {label: d} record."""
    return [int(part.get(l, 1)) for l in unique_labels(spec)]


def _uniform_part(vertices: List[Vertex], split: Dict[str, int]) -> Dict[str, Dict[str, int]]:
    """Apply the same {label: d} to every einsum vertex, keeping only labels the vertex has."""
    out = {}
    for v in vertices:
        if v.is_input:
            continue
        labs = unique_labels(v.spec)
        out[v.name] = {l: d for l, d in split.items() if l in labs}
    return out


# ----------------------------------------------------------------------------------------------
# C1: single fp32 matmul, contracted label split in two
# ----------------------------------------------------------------------------------------------
def config1(dims=None) -> Workload:
    dm = {"i": 256, "j": 256, "k": 256}
    dm.update(dims or {})
    vs = [
        Vertex("X", "f32", bound=(dm["i"], dm["j"]), recipe={"dist": "uniform"}),
        Vertex("Y", "f32", bound=(dm["j"], dm["k"]), recipe={"dist": "uniform"}),
        Vertex("Z", "f32", spec="ij,jk->ik", inputs=("X", "Y")),
    ]
    parts = {}
    for d in [(2, 2, 2), (1, 1, 1), (8, 1, 1), (1, 8, 1), (1, 1, 8), (4, 2, 1), (2, 1, 4), (1, 2, 4), (4, 4, 4)]:
        parts["d%d%d%d" % d] = {"Z": {"i": d[0], "j": d[1], "k": d[2]}}
    return Workload("c1_matmul_f32", SEED_BASE + 1, vs, ["Z"], parts, dm)


# ----------------------------------------------------------------------------------------------
# C2: matrix chain (A.B).C, bf16 storage, fp32 accumulation
# ----------------------------------------------------------------------------------------------
def config2(dims=None) -> Workload:
    dm = {"i": 8192, "j": 8192, "k": 8192, "l": 8192}
    dm.update(dims or {})
    std = 1.0 / (8192.0 ** 0.5)   # second parameter of N(0, 1/sqrt(8192)) read as the std-dev
    vs = [
        Vertex("A", "bf16", bound=(dm["i"], dm["j"]), recipe={"dist": "normal", "std": std}),
        Vertex("B", "bf16", bound=(dm["j"], dm["k"]), recipe={"dist": "normal", "std": std}),
        Vertex("C", "bf16", bound=(dm["k"], dm["l"]), recipe={"dist": "normal", "std": std}),
        Vertex("AB", "bf16", spec="ij,jk->ik", inputs=("A", "B")),
        Vertex("ABC", "f32", spec="ik,kl->il", inputs=("AB", "C")),
    ]

    def both(d):
        return {"AB": {"i": d[0], "j": d[1], "k": d[2]}, "ABC": {"i": d[0], "k": d[1], "l": d[2]}}

    parts = {
        # the mandated pair: first product cut (2,2,2), second cut (1,2,4); AB is produced with
        # d_Z = [2,2] and consumed with d_X = [1,2], so a repartition sits between them
        "mix": {"AB": {"i": 2, "j": 2, "k": 2}, "ABC": {"i": 1, "k": 2, "l": 4}},
        "d222": both((2, 2, 2)),
        "d124": both((1, 2, 4)),
        "sqrt214": both((2, 1, 4)),
        "sqrt412": both((4, 1, 2)),
        "splitk8": both((1, 8, 1)),
        "rows8": both((8, 1, 1)),
        "whole": both((1, 1, 1)),
    }
    return Workload("c2_matrix_chain_bf16", SEED_BASE + 2, vs, ["ABC"], parts, dm)


# ----------------------------------------------------------------------------------------------
# C3: one FFNN training step (forward, softmax cross-entropy, backward to dW1/dW2)
# ----------------------------------------------------------------------------------------------
def config3(dims=None) -> Workload:
    dm = {"b": 4096, "f": 8192, "h": 4096, "c": 1024}
    dm.update(dims or {})
    B = dm["b"]
    vs = [
        Vertex("X", "bf16", bound=(dm["b"], dm["f"]), recipe={"dist": "normal", "std": 1.0}),
        Vertex("W1", "bf16", bound=(dm["f"], dm["h"]), recipe={"dist": "normal", "std": 0.02}),
        Vertex("W2", "bf16", bound=(dm["h"], dm["c"]), recipe={"dist": "normal", "std": 0.02}),
        Vertex("Y", "bf16", bound=(dm["b"], dm["c"]), recipe={"dist": "onehot"}),
        Vertex("H1", "bf16", spec="bf,fh->bh", inputs=("X", "W1")),
        Vertex("A1", "bf16", spec="bh->bh", otimes="relu", oplus="none", inputs=("H1",)),
        Vertex("L", "f32", spec="bh,hc->bc", inputs=("A1", "W2")),
        # row softmax as four einsums (max, exp of difference, sum, divide)
        Vertex("Cmax", "f32", spec="bc->b", otimes="ident", oplus="max", inputs=("L",)),
        Vertex("E", "f32", spec="bc,b->bc", otimes="exp_sub", oplus="none", inputs=("L", "Cmax")),
        Vertex("S", "f32", spec="bc->b", otimes="ident", oplus="sum", inputs=("E",)),
        Vertex("P", "f32", spec="bc,b->bc", otimes="div", oplus="none", inputs=("E", "S")),
        # cross-entropy in log-softmax form: -(1/B) sum_bc Y * ((L - C) - log S)
        Vertex("D", "f32", spec="bc,b->bc", otimes="sub", oplus="none", inputs=("L", "Cmax")),
        Vertex("logS", "f32", spec="b->b", otimes="log", oplus="none", inputs=("S",)),
        Vertex("logP", "f32", spec="bc,b->bc", otimes="sub", oplus="none", inputs=("D", "logS")),
        Vertex("loss", "f32", spec="bc,bc->", otimes="mul", oplus="sum", alpha=-1.0 / B, inputs=("Y", "logP")),
        # backward
        Vertex("dL", "bf16", spec="bc,bc->bc", otimes="sub", oplus="none", alpha=1.0 / B, inputs=("P", "Y")),
        Vertex("dW2", "f32", spec="bh,bc->hc", inputs=("A1", "dL")),
        Vertex("dA1", "bf16", spec="bc,hc->bh", inputs=("dL", "W2")),
        Vertex("dH1", "bf16", spec="bh,bh->bh", otimes="relu_grad", oplus="none", inputs=("dA1", "H1")),
        Vertex("dW1", "f32", spec="bf,bh->fh", inputs=("X", "dH1")),
    ]
    parts = {
        "batch8": _uniform_part(vs, {"b": 8}),             # data parallel: dW1/dW2 are 8 partial sums
        "hidden8": {},
        "mixed": {},
        "whole": _uniform_part(vs, {}),
    }
    # hidden-split: h:8 where the vertex has h, class label c:8 elsewhere (split softmax reductions)
    hid, mix = {}, {}
    for v in vs:
        if v.is_input:
            continue
        labs = unique_labels(v.spec)
        if "h" in labs:
            hid[v.name] = {"h": 8}
            mix[v.name] = {"b": 2, "h": 4}
        elif "c" in labs:
            hid[v.name] = {"c": 8}
            mix[v.name] = {"b": 2, "c": 4}
        else:
            hid[v.name] = {"b": 8}
            mix[v.name] = {"b": 8}
    parts["hidden8"] = hid
    parts["mixed"] = mix
    return Workload("c3_ffnn_step_bf16", SEED_BASE + 3, vs, ["loss", "dW1", "dW2"], parts, dm)


# ----------------------------------------------------------------------------------------------
# C4: decoder block: multi-head causal attention (paper Section 3, with a batch label) + SwiGLU
# ----------------------------------------------------------------------------------------------
def config4(dims=None) -> Workload:
    dm = {"b": 4, "s": 2048, "a": 4096, "h": 32, "d": 128, "f": 11008}
    dm.update(dims or {})
    b, s, a, h, d, f = (dm[k] for k in "bsahdf")
    w = {"dist": "normal", "std": 0.02}
    vs = [
        Vertex("X", "bf16", bound=(b, s, a), recipe={"dist": "normal", "std": 1.0}),
        Vertex("Wq", "bf16", bound=(a, h, d), recipe=w),
        Vertex("Wk", "bf16", bound=(a, h, d), recipe=w),
        Vertex("Wv", "bf16", bound=(a, h, d), recipe=w),
        Vertex("Wo", "bf16", bound=(a, h, d), recipe=w),
        Vertex("M", "f32", bound=(s, s), recipe={"dist": "causal_mask"}),
        Vertex("Wg", "bf16", bound=(a, f), recipe=w),
        Vertex("Wu", "bf16", bound=(a, f), recipe=w),
        Vertex("Wd", "bf16", bound=(f, a), recipe=w),
        Vertex("Q", "bf16", spec="bsa,ahd->bshd", inputs=("X", "Wq")),
        Vertex("K", "bf16", spec="bta,ahd->bthd", inputs=("X", "Wk")),
        Vertex("V", "bf16", spec="bta,ahd->bthd", inputs=("X", "Wv")),
        Vertex("T1", "bf16", spec="bshd,bthd->bhst", inputs=("Q", "K")),
        Vertex("T2", "bf16", spec="bhst,st->bhst", otimes="add", oplus="none", alpha=1.0 / (d ** 0.5),
               inputs=("T1", "M")),
        Vertex("Cmax", "f32", spec="bhst->bhs", otimes="ident", oplus="max", inputs=("T2",)),
        Vertex("E", "bf16", spec="bhst,bhs->bhst", otimes="exp_sub", oplus="none", inputs=("T2", "Cmax")),
        Vertex("S", "f32", spec="bhst->bhs", otimes="ident", oplus="sum", inputs=("E",)),
        Vertex("P", "bf16", spec="bhst,bhs->bhst", otimes="div", oplus="none", inputs=("E", "S")),
        Vertex("O", "bf16", spec="bhst,bthd->bshd", inputs=("P", "V")),
        Vertex("Yatt", "bf16", spec="bshd,ahd->bsa", inputs=("O", "Wo")),
        Vertex("G", "bf16", spec="bsa,af->bsf", inputs=("Yatt", "Wg")),
        Vertex("U", "bf16", spec="bsa,af->bsf", inputs=("Yatt", "Wu")),
        Vertex("Hh", "bf16", spec="bsf,bsf->bsf", otimes="silu_mul", oplus="none", inputs=("G", "U")),
        Vertex("Out", "f32", spec="bsf,fa->bsa", inputs=("Hh", "Wd")),
    ]
    heads, seq, tsp = {}, {}, {}
    for v in vs:
        if v.is_input:
            continue
        labs = unique_labels(v.spec)
        # Megatron-like: heads split through attention, FFN hidden label split in the MLP
        if "h" in labs:
            heads[v.name] = {"h": 8}
        elif "f" in labs:
            heads[v.name] = {"f": 8}
        else:
            heads[v.name] = {"s": 8}
        # "sequence": split the sequence label everywhere (t on the key/value side projections)
        seq[v.name] = {"s": 8} if "s" in labs else {"t": 8}
        # split the key label t through the softmax: max- and sum-aggregation of partial rows
        if "t" in labs:
            tsp[v.name] = {"t": 8}
        elif "f" in labs:
            tsp[v.name] = {"f": 8}
        else:
            tsp[v.name] = {"s": 8}
    parts = {"heads8": heads, "seq8": seq, "tsplit8": tsp, "whole": _uniform_part(vs, {})}
    return Workload("c4_decoder_block_bf16", SEED_BASE + 4, vs, ["Out"], parts, dm)


# ----------------------------------------------------------------------------------------------
# C5: large contraction with the reduction label split 16 ways
# ----------------------------------------------------------------------------------------------
def config5(dims=None) -> Workload:
    dm = {"i": 64, "j": 1024, "k": 16384, "l": 4096}
    dm.update(dims or {})
    vs = [
        Vertex("X", "bf16", bound=(dm["i"], dm["j"], dm["k"]), recipe={"dist": "uniform"}),
        Vertex("Y", "bf16", bound=(dm["k"], dm["l"]), recipe={"dist": "uniform"}),
        Vertex("Z", "f32", spec="ijk,kl->ijl", inputs=("X", "Y")),
    ]
    parts = {
        "k16": {"Z": {"k": 16}},
        "k1": {"Z": {}},
        "k2": {"Z": {"k": 2}},
        "k4": {"Z": {"k": 4}},
        "k8": {"Z": {"k": 8}},
        "i2k8": {"Z": {"i": 2, "k": 8}},
    }
    return Workload("c5_split_reduction_bf16", SEED_BASE + 5, vs, ["Z"], parts, dm)


# ----------------------------------------------------------------------------------------------
# C6: the matrix chain of the paper's first experiment, (A x B) + (C x (D x E)), in its skewed version:
# for a scale s, A is s x .1s, B .1s x s, C s x .1s, D .1s x 10s, E 10s x s (the square version is config 2's shape)
# ----------------------------------------------------------------------------------------------
def config6(dims=None) -> Workload:
    dm = {"i": 10240, "j": 1024, "k": 10240, "m": 1024, "n": 102400}
    dm.update(dims or {})
    sd = lambda k: {"dist": "normal", "std": float(k) ** -0.25}      # a product over k of two such factors has unit variance
    vs = [
        Vertex("A", "bf16", bound=(dm["i"], dm["j"]), recipe=sd(dm["j"])),
        Vertex("B", "bf16", bound=(dm["j"], dm["k"]), recipe=sd(dm["j"])),
        Vertex("C", "bf16", bound=(dm["i"], dm["m"]), recipe={"dist": "normal", "std": float(dm["m"]) ** -0.5}),
        Vertex("D", "bf16", bound=(dm["m"], dm["n"]), recipe=sd(dm["n"])),
        Vertex("E", "bf16", bound=(dm["n"], dm["k"]), recipe=sd(dm["n"])),
        Vertex("AB", "bf16", spec="ij,jk->ik", inputs=("A", "B")),
        Vertex("DE", "bf16", spec="mn,nk->mk", inputs=("D", "E")),
        Vertex("CDE", "bf16", spec="im,mk->ik", inputs=("C", "DE")),
        Vertex("Z", "f32", spec="ik,ik->ik", inputs=("AB", "CDE"), otimes="add", oplus="none"),
    ]
    parts = {
        # the "3D" cut of every product, the sum cut like the products' outputs
        "d222": {"AB": {"i": 2, "j": 2, "k": 2}, "DE": {"m": 2, "n": 2, "k": 2}, "CDE": {"i": 2, "m": 2, "k": 2}, "Z": {"i": 2, "k": 4}},
        # square-root style: outputs cut 2 x 4, nothing aggregated
        "sqrt": {"AB": {"i": 2, "k": 4}, "DE": {"m": 2, "k": 4}, "CDE": {"i": 2, "k": 4}, "Z": {"i": 2, "k": 4}},
        # the long contraction of D x E cut 8 ways, the two summands cut differently (a repartition into the sum)
        "splitn8": {"AB": {"i": 4, "k": 2}, "DE": {"n": 8}, "CDE": {"i": 2, "k": 4}, "Z": {"i": 8}},
        "whole": {},
    }
    return Workload("c6_skewed_chain_bf16", SEED_BASE + 6, vs, ["Z"], parts, dm)


# ----------------------------------------------------------------------------------------------
# C7: the paper's two extended examples: squared L2 and L-infinity distance between the rows of X and the
# columns of Y (scalar function (x - y)^2 with sum, |x - y| with max)
# ----------------------------------------------------------------------------------------------
def config7(dims=None) -> Workload:
    dm = {"i": 8192, "j": 1024, "k": 8192}
    dm.update(dims or {})
    vs = [
        Vertex("X", "f32", bound=(dm["i"], dm["j"]), recipe={"dist": "uniform"}),
        Vertex("Y", "f32", bound=(dm["j"], dm["k"]), recipe={"dist": "uniform"}),
        Vertex("Xh", "bf16", bound=(dm["i"], dm["j"]), recipe={"dist": "uniform"}),
        Vertex("Yh", "bf16", bound=(dm["k"], dm["j"]), recipe={"dist": "uniform"}),
        Vertex("L2", "f32", spec="ij,jk->ik", inputs=("X", "Y"), otimes="sqdiff"),
        Vertex("Linf", "f32", spec="ij,jk->ik", inputs=("X", "Y"), otimes="absdiff", oplus="max"),
        Vertex("L2h", "f32", spec="ij,kj->ik", inputs=("Xh", "Yh"), otimes="sqdiff"),
        Vertex("Linfh", "bf16", spec="ij,kj->ik", inputs=("Xh", "Yh"), otimes="absdiff", oplus="max"),
    ]

    def all4(d):
        return {n: dict(d) for n in ("L2", "Linf", "L2h", "Linfh")}

    parts = {"d222": all4({"i": 2, "j": 2, "k": 2}), "ik8": all4({"i": 2, "k": 4}), "j8": all4({"j": 8}), "whole": {}}
    return Workload("c7_distances", SEED_BASE + 7, vs, ["L2", "Linf", "L2h", "Linfh"], parts, dm)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5, 6: config6, 7: config7}

# Scaled-down shapes that the CPU oracle finishes in seconds while every block still spans
# several kernel tiles with ragged tails.
SMALL_DIMS = {
    1: {"i": 256, "j": 256, "k": 256},
    2: {"i": 384, "j": 512, "k": 320, "l": 448},
    3: {"b": 256, "f": 384, "h": 320, "c": 128},
    4: {"b": 2, "s": 128, "a": 256, "h": 8, "d": 32, "f": 704},
    5: {"i": 4, "j": 48, "k": 1024, "l": 192},
    6: {"i": 320, "j": 40, "k": 288, "m": 48, "n": 2560},
    7: {"i": 200, "j": 152, "k": 136},
}


def build_config(n: int, dims=None, small: bool = False) -> Workload:
    dm = dict(SMALL_DIMS[n]) if small else {}
    dm.update(dims or {})
    return CONFIGS[n](dm)
