"""planner_ref: the paper's cost model and the EinDecomp labelling, written out plainly.  TEST INFRASTRUCTURE ONLY.

Follows Sections 6-8 of the paper:
  * Section 6: a partitioning vector d (one entry per unique label, co-partitioned labels share it) gives
    N = prod d join results; `viable` lists the power-of-two vectors with exactly p of them.
  * Section 7: the cost of a labelled vertex is an upper bound on the floating point numbers moved:
    into the join p (n_X + n_Y), into the aggregation (p / n_agg)(n_agg - 1) n_Z, and between a producer and
    a consumer with different partitionings (n_c/n_int - 1)(n/n_c)(n_c + n_p) [+ n_p n/n_c if n_p != n_int].
  * Section 8.2-8.3: dynamic programming over a topological order with the table M[v, d_Z].
  * Section 8.4: graphs with shared intermediate results are cut into paths, longest first, and each path is
    optimised on its own; inputs to a path from outside it cost nothing.

Readings taken where the text leaves a choice or contradicts itself:
  * the join-cost example prints "8 x (16 + 16)" for d = [4,1,1,4], whose join has 16 results; the formula
    p (n_X + n_Y) with p = N(d) = 16 is taken (n_X = n_Y = 16 as printed);
  * in the repartition cost the consumer's sub-tensor size uses the consumer's partitioning and n is the number
    of elements of the tensor (prod b), which is what reproduces the printed total of 320; the two printed
    summands 128 + 192 do not match the formula's 32 + 288 and are not pinned;
  * in the recurrence the repartition is from the producer's output partitioning (the key of M) to what the
    consumer's d demands of that operand, d[l_X; l_XY];
  * a vertex with one input pays p n_X into the join (nothing is said about them);
  * every entry of d must divide its label's bound (the paper's examples all do); when no vector with p
    results exists for a vertex (bounds too small) p is halved for that vertex until one does;
  * ties are broken towards the vector enumerated first (exponents in lexicographic order over the unique
    labels in first-appearance order); any of the tied labellings is a correct answer;
  * paths: among the vertices not yet labelled, the longest chain of producer -> consumer edges (ties: the
    one whose vertex ids, in creation order, are lexicographically smallest).

Pins (tests/test_planner_oracle.py): the printed values of Sections 7 and 8.1, closed forms of the re-partition cost,
exhaustive search for the dynamic programme, and for the path heuristic of Section 8.4 (the paper prints no example)
a graph with a shared result whose paths, per-path tables M and final vectors were worked out by hand from the
formulas of Section 7 and are written into the test as literals.  Nothing in this file is unpinned.
"""
from __future__ import annotations

import itertools
import math
from fractions import Fraction
from typing import Dict, List, Optional, Sequence, Tuple

Labels = Dict[str, int]          # label -> number of slices


def split_spec(spec: str) -> Tuple[List[List[str]], List[str]]:
    lhs, rhs = spec.split("->")
    return [list(s) for s in lhs.split(",")], list(rhs)


def unique_labels(ins: Sequence[Sequence[str]]) -> List[str]:
    out: List[str] = []
    for s in ins:
        for l in s:
            if l not in out:
                out.append(l)
    return out


# ---------------------------------------------------------------------------- Section 6 / 8.1
def viable(spec: str, bounds: Dict[str, int], p: int) -> List[Labels]:
    """Power-of-two partitioning vectors with exactly p join results whose entries divide the bounds."""
    ins, _ = split_spec(spec)
    uniq = unique_labels(ins)
    n = int(round(math.log2(p)))
    if 2 ** n != p:
        raise ValueError("p must be a power of two")
    out = []
    for combo in itertools.product(range(n + 1), repeat=len(uniq)):
        if sum(combo) != n:
            continue
        d = {l: 2 ** e for l, e in zip(uniq, combo)}
        if all(bounds[l] % d[l] == 0 for l in uniq):
            out.append(d)
    return out


def viable_or_fewer(spec: str, bounds: Dict[str, int], p: int) -> List[Labels]:
    while p >= 1:
        v = viable(spec, bounds, p)
        if v:
            return v
        p //= 2
    raise ValueError("no partitioning")


# ---------------------------------------------------------------------------- Section 7
def cost_join(spec: str, bounds: Dict[str, int], d: Labels) -> int:
    ins, _ = split_spec(spec)
    p = math.prod(d[l] for l in unique_labels(ins))
    per_input = [math.prod(bounds[l] // d[l] for l in s) for s in ins]
    return p * sum(per_input)


def cost_agg(spec: str, bounds: Dict[str, int], d: Labels) -> int:
    ins, lz = split_spec(spec)
    uniq = unique_labels(ins)
    p = math.prod(d[l] for l in uniq)
    n_agg = math.prod(d[l] for l in uniq if l not in lz)
    n_z = math.prod(bounds[l] // d[l] for l in lz)
    return (p // n_agg) * (n_agg - 1) * n_z


def cost_repart(d_consumer: Sequence[int], d_producer: Sequence[int], bound: Sequence[int]) -> Fraction:
    ext_p = [b // d for b, d in zip(bound, d_producer)]
    ext_c = [b // d for b, d in zip(bound, d_consumer)]
    n_p = math.prod(ext_p)
    n_c = math.prod(ext_c)
    n_int = math.prod(min(a, b) for a, b in zip(ext_p, ext_c))
    n = math.prod(bound)
    cost = (Fraction(n_c, n_int) - 1) * Fraction(n, n_c) * (n_c + n_p)
    if n_p != n_int:
        cost += n_p * Fraction(n, n_c)
    return cost


# ---------------------------------------------------------------------------- graphs
class PVertex:
    """One vertex for the planner: name, spec (None for an input), ordered inputs, bound of its output."""

    def __init__(self, name: str, spec: Optional[str], inputs: Sequence[str], bound: Sequence[int]):
        self.name, self.spec, self.inputs, self.bound = name, spec, list(inputs), [int(b) for b in bound]


def from_workload(w) -> List[PVertex]:
    """Vertices of a synthetic workload; an einsum vertex's bound is b_Z = b_XY[l_Z; l_XY] (Section 3)."""
    out: List[PVertex] = []
    bound: Dict[str, List[int]] = {}
    for v in w.vertices:
        if v.is_input:
            bound[v.name] = [int(x) for x in v.bound]
            out.append(PVertex(v.name, None, [], bound[v.name]))
            continue
        ins, lz = split_spec(v.spec)
        lb: Dict[str, int] = {}
        for s_, name in zip(ins, v.inputs):
            for l, e in zip(s_, bound[name]):
                lb[l] = e
        bound[v.name] = [lb[l] for l in lz]
        out.append(PVertex(v.name, v.spec, v.inputs, bound[v.name]))
    return out


def label_bounds(g: Dict[str, PVertex], v: PVertex) -> Dict[str, int]:
    ins, _ = split_spec(v.spec)
    b: Dict[str, int] = {}
    for s, name in zip(ins, v.inputs):
        for l, e in zip(s, g[name].bound):
            b[l] = e
    return b


def vertex_cost(g: Dict[str, PVertex], v: PVertex, d: Labels, producer_dz: Dict[str, Optional[List[int]]]) -> Fraction:
    """join + aggregation + repartition of every operand whose producer's output partitioning is given."""
    b = label_bounds(g, v)
    ins, _ = split_spec(v.spec)
    c = Fraction(cost_join(v.spec, b, d) + cost_agg(v.spec, b, d))
    for s, name in zip(ins, v.inputs):
        dz = producer_dz.get(name)
        if dz is not None:
            c += cost_repart([d[l] for l in s], dz, g[name].bound)
    return c


def out_partition(v: PVertex, d: Labels) -> List[int]:
    _, lz = split_spec(v.spec)
    return [d[l] for l in lz]


def labelling_cost(vs: Sequence[PVertex], labels: Dict[str, Labels]) -> Fraction:
    """Total cost of a fully labelled graph, every producer -> consumer edge included."""
    g = {v.name: v for v in vs}
    total = Fraction(0)
    for v in vs:
        if v.spec is None:
            continue
        prod_dz = {n: (None if g[n].spec is None else out_partition(g[n], labels[n])) for n in v.inputs}
        total += vertex_cost(g, v, labels[v.name], prod_dz)
    return total


def brute_force(vs: Sequence[PVertex], p: int) -> Tuple[Fraction, Dict[str, Labels]]:
    """The definition: the cheapest of all labellings (tiny graphs only)."""
    g = {v.name: v for v in vs}
    ein = [v for v in vs if v.spec is not None]
    choices = [viable_or_fewer(v.spec, label_bounds(g, v), p) for v in ein]
    best: Optional[Tuple[Fraction, Dict[str, Labels]]] = None
    for combo in itertools.product(*choices):
        labels = {v.name: d for v, d in zip(ein, combo)}
        c = labelling_cost(vs, labels)
        if best is None or c < best[0]:
            best = (c, labels)
    assert best is not None
    return best


# ---------------------------------------------------------------------------- Section 8.2-8.3
def dp_chain(g: Dict[str, PVertex], order: Sequence[PVertex], edges, p: int):
    """The table M over `order` (a topological order).  An operand contributes M and a repartition only when the
    edge (producer, consumer) is in `edges`; returns M[v] = {d_Z: (cost, d, {producer: its d_Z})}."""
    M: Dict[str, Dict[Tuple[int, ...], Tuple[Fraction, Labels, Dict[str, Tuple[int, ...]]]]] = {}
    for v in order:
        b = label_bounds(g, v)
        ins, _ = split_spec(v.spec)
        table: Dict[Tuple[int, ...], Tuple[Fraction, Labels, Dict[str, Tuple[int, ...]]]] = {}
        for d in viable_or_fewer(v.spec, b, p):
            c = Fraction(cost_join(v.spec, b, d) + cost_agg(v.spec, b, d))
            picks: Dict[str, Tuple[int, ...]] = {}
            for s, name in zip(ins, v.inputs):
                if g[name].spec is None or (name, v.name) not in edges:
                    continue
                assert name not in picks, "a producer feeding both operands of one vertex is not handled"
                want = [d[l] for l in s]
                best = None
                for dz, (cz, _, _) in M[name].items():
                    t = cz + cost_repart(want, list(dz), g[name].bound)
                    if best is None or t < best[0]:
                        best = (t, dz)
                c += best[0]
                picks[name] = best[1]
            key = tuple(out_partition(v, d))
            if key not in table or c < table[key][0]:
                table[key] = (c, d, picks)
        M[v.name] = table
    return M


def backtrack(g, M, last: str, labels: Dict[str, Labels]) -> Fraction:
    best_cost = min(c for c, _, _ in M[last].values())
    best_key = next(k for k, (c, _, _) in M[last].items() if c == best_cost)     # ties: the first one entered

    def walk(name: str, key: Tuple[int, ...]):
        c, d, picks = M[name][key]
        labels[name] = d
        for n, k in picks.items():
            walk(n, k)

    walk(last, best_key)
    return best_cost


def consumers_of(vs: Sequence[PVertex]) -> Dict[str, List[str]]:
    out: Dict[str, List[str]] = {v.name: [] for v in vs}
    for v in vs:
        for n in v.inputs:
            if v.name not in out[n]:
                out[n].append(v.name)
    return out


def eindecomp_tree(vs: Sequence[PVertex], p: int) -> Tuple[Fraction, Dict[str, Labels]]:
    """Sections 8.2-8.3: exact when no non-input vertex has two consumers and there is one output vertex."""
    g = {v.name: v for v in vs}
    cons = consumers_of(vs)
    ein = [v for v in vs if v.spec is not None]
    assert all(len(cons[v.name]) <= 1 for v in ein), "a non-input vertex has two consumers"
    sinks = [v for v in ein if not cons[v.name]]
    assert len(sinks) == 1, "one output vertex expected"
    M = dp_chain(g, ein, {(n, v.name) for v in ein for n in v.inputs}, p)
    labels: Dict[str, Labels] = {}
    cost = backtrack(g, M, sinks[0].name, labels)
    return cost, labels


# ---------------------------------------------------------------------------- Section 8.4
def longest_path(vs: Sequence[PVertex], unlabelled: Sequence[str]) -> List[str]:
    g = {v.name: v for v in vs}
    idx = {v.name: i for i, v in enumerate(vs)}
    todo = [v.name for v in vs if v.name in unlabelled]
    best_to: Dict[str, List[str]] = {}
    for n in todo:                                  # creation order is a topological order
        cand = [[n]]
        for u in g[n].inputs:
            if u in best_to:
                cand.append(best_to[u] + [n])
        best_to[n] = max(cand, key=lambda pth: (len(pth), [-idx[x] for x in pth]))
    return max(best_to.values(), key=lambda pth: (len(pth), [-idx[x] for x in pth]))


def eindecomp_paths(vs: Sequence[PVertex], p: int) -> Dict[str, Labels]:
    g = {v.name: v for v in vs}
    labels: Dict[str, Labels] = {}
    unlabelled = [v.name for v in vs if v.spec is not None]
    while unlabelled:
        path = longest_path(vs, unlabelled)
        M = dp_chain(g, [g[n] for n in path], set(zip(path[:-1], path[1:])), p)
        backtrack(g, M, path[-1], labels)
        unlabelled = [n for n in unlabelled if n not in path]
    return labels
