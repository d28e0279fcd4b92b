"""Pins of the planner oracle (cost model of Section 7, enumeration and dynamic programme of Section 8 of the paper)."""
import itertools
import math
import os
from fractions import Fraction

import pytest

from oracle import planner_ref as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bookkeeping.txt")


def golden(prefix):
    rows = []
    for line in open(GOLDEN):
        if line.startswith(prefix + " "):
            rows.append(line[len(prefix) + 1:].strip())
    return rows


MM = "ij,jk->ik"
B8 = {"i": 8, "j": 8, "k": 8}


def full(d4):
    """the paper's 4-entry vector over l_XY = [i,j,j,k] -> per label"""
    assert d4[1] == d4[2]
    return {"i": d4[0], "j": d4[1], "k": d4[3]}


def test_join_cost_of_the_printed_example():
    (row,) = golden("subbound")
    d = [int(x) for x in row.split("d=")[1].split()[0].split(",")]
    lab = full(d)
    assert [B8[l] // lab[l] for l in "ij"] == [2, 8] and [B8[l] // lab[l] for l in "jk"] == [8, 2]
    # 16 join results, each receiving a 16-element block of X and one of Y
    assert P.cost_join(MM, B8, lab) == 16 * (16 + 16)


def test_aggregation_cost_of_the_printed_example():
    (row,) = golden("aggcost")
    want = int(row.split("cost=")[1])
    d = [int(x) for x in row.split("d=")[1].split()[0].split(",")]
    assert want == 64 and P.cost_agg(MM, B8, full(d)) == want
    assert P.cost_agg(MM, B8, full([4, 1, 1, 4])) == 0          # the shared label is not cut: nothing to aggregate


def test_repartition_cost_of_the_printed_example():
    (row,) = golden("repart")
    f = dict(kv.split("=") for kv in row.replace("->", "").split())
    bound = [int(x) for x in f["bound"].split(",")]
    prod = [int(x) for x in f["producer"].split(",")]
    cons = [int(x) for x in f["consumer"].split(",")]
    assert math.prod(b // d for b, d in zip(bound, prod)) == int(f["np"])
    assert math.prod(b // d for b, d in zip(bound, cons)) == int(f["nc"])
    assert P.cost_repart(cons, prod, bound) == int(f["cost"]) == 320


def test_repartition_cost_special_cases():
    for d in ([1, 1], [2, 4], [8, 8]):
        assert P.cost_repart(d, d, [8, 8]) == 0                  # same cut: nothing moves
    # consumer blocks inside producer blocks: every producer block is sent once to each place a piece of it is cut out
    assert P.cost_repart([4, 4], [2, 2], [8, 8]) == 16 * 16     # n_p = 16, n/n_c = 16 consumer blocks
    # producer blocks inside consumer blocks, 4 per consumer block: 3 further hops of (n_c + n_p) each
    assert P.cost_repart([1, 2], [2, 4], [8, 8]) == 3 * 2 * (32 + 8)


def test_viable_lists_the_papers_vectors_and_counts_balls_in_buckets():
    got = {(d["i"], d["j"], d["j"], d["k"]) for d in P.viable(MM, B8, 8)}
    printed = {tuple(int(x) for x in r.split("->")[0].strip().split(",")) for r in golden("viable")}
    assert len(printed) == 8 and printed <= got
    assert got - printed == {(2, 4, 4, 1), (1, 4, 4, 2)} and len(got) == math.comb(3 + 3 - 1, 3)
    assert all(d["i"] * d["j"] * d["k"] == 8 for d in P.viable(MM, B8, 8))
    # N = 10 doublings over D = 6 unique labels
    big = {l: 1 << 10 for l in "abcdef"}
    assert len(P.viable("abcd,cdef->abef", big, 1 << 10)) == 3003
    # entries must divide the bounds
    assert all(d["j"] <= 2 for d in P.viable(MM, {"i": 8, "j": 2, "k": 8}, 8))


def chain(n_mats, dims, unary_tail=False):
    """A_0 x A_1 x ... as a left-deep chain; dims[i] x dims[i+1] matrices."""
    vs = [P.PVertex(f"A{i}", None, [], [dims[i], dims[i + 1]]) for i in range(n_mats)]
    prev = "A0"
    for i in range(1, n_mats):
        name = f"M{i}"
        vs.append(P.PVertex(name, "ij,jk->ik", [prev, f"A{i}"], [dims[0], dims[i + 1]]))
        prev = name
    if unary_tail:
        vs.append(P.PVertex("R", "ik->i", [prev], [dims[0]]))
    return vs


def tree():
    """(A x B) x (C x D) followed by a row sum"""
    vs = [P.PVertex(n, None, [], [8, 8]) for n in "ABCD"]
    vs.append(P.PVertex("AB", "ij,jk->ik", ["A", "B"], [8, 8]))
    vs.append(P.PVertex("CD", "kl,lm->km", ["C", "D"], [8, 8]))
    vs.append(P.PVertex("Z", "ik,km->im", ["AB", "CD"], [8, 8]))
    return vs


@pytest.mark.parametrize("vs,p", [(chain(3, [8, 8, 8, 8]), 4), (chain(3, [16, 4, 32, 8]), 8), (chain(4, [8, 16, 4, 8, 8]), 4),
                                  (chain(3, [8, 8, 8, 8], unary_tail=True), 4), (tree(), 4)])
def test_dynamic_programme_finds_the_exhaustive_optimum(vs, p):
    cost, labels = P.eindecomp_tree(vs, p)
    want, _ = P.brute_force(vs, p)
    assert cost == want
    assert P.labelling_cost(vs, labels) == cost                  # the labelling it returns really costs that
    g = {v.name: v for v in vs}
    for v in vs:
        if v.spec is not None:
            d = labels[v.name]
            assert math.prod(d.values()) == p and all(P.label_bounds(g, v)[l] % d[l] == 0 for l in d)


def test_single_vertex_optimum_is_the_cheapest_viable_vector():
    vs = chain(2, [64, 8, 64])
    cost, labels = P.eindecomp_tree(vs, 16)
    b = {"i": 64, "j": 8, "k": 64}
    assert cost == min(P.cost_join(MM, b, d) + P.cost_agg(MM, b, d) for d in P.viable(MM, b, 16))
    assert labels["M1"] == {"i": 4, "j": 1, "k": 4}              # the square cut of the output, nothing aggregated


def diamond():
    """one product feeding two consumers whose results are added: needs the path decomposition"""
    vs = [P.PVertex(n, None, [], [8, 8]) for n in "ABC"]
    vs.append(P.PVertex("AB", "ij,jk->ik", ["A", "B"], [8, 8]))
    vs.append(P.PVertex("L", "ik,kl->il", ["AB", "C"], [8, 8]))
    vs.append(P.PVertex("R", "ik,kl->il", ["AB", "B"], [8, 8]))
    vs.append(P.PVertex("S", "il,il->il", ["L", "R"], [8, 8]))
    return vs


def test_path_decomposition_labels_everything_validly_and_is_no_better_than_the_optimum():
    vs = diamond()
    assert P.longest_path(vs, ["AB", "L", "R", "S"]) == ["AB", "L", "S"]
    assert P.longest_path(vs, ["R"]) == ["R"]
    labels = P.eindecomp_paths(vs, 4)
    assert set(labels) == {"AB", "L", "R", "S"}
    assert all(math.prod(d.values()) == 4 for d in labels.values())
    best, _ = P.brute_force(vs, 4)
    assert P.labelling_cost(vs, labels) >= best
    # on a graph that is one path the heuristic is the dynamic programme
    c = chain(4, [8, 16, 4, 8, 8])
    assert P.labelling_cost(c, P.eindecomp_paths(c, 4)) == P.eindecomp_tree(c, 4)[0]


# ------------------------------------------------------------------ Section 8.4 worked by hand
def shared_result_graph():
    """T = X W feeds both U = relu(T) and V = T W2; S contracts U with V over the rows.  X is 8 x 4, W 4 x 4, W2 4 x 16."""
    return [P.PVertex("X", None, [], [8, 4]), P.PVertex("W", None, [], [4, 4]), P.PVertex("W2", None, [], [4, 16]),
            P.PVertex("T", "ij,jk->ik", ["X", "W"], [8, 4]),
            P.PVertex("U", "ik->ik", ["T"], [8, 4]),
            P.PVertex("V", "ik,kl->il", ["T", "W2"], [8, 16]),
            P.PVertex("S", "ik,il->kl", ["U", "V"], [4, 16])]


# Worked with pencil from the formulas of Section 7 for p = 2 (every vector has one entry equal to 2).
#   T (i=8, j=4, k=4), both inputs are graph inputs:
#     k cut: n_X = 8*4 = 32, n_Y = 4*2 = 8, join 2*(32+8) = 80, nothing aggregated          -> d_Z [1,2]: 80
#     j cut: n_X = 8*2 = 16, n_Y = 2*4 = 8, join 2*24 = 48, n_agg = 2, n_Z = 32, agg 32     -> d_Z [1,1]: 80
#     i cut: n_X = 4*4 = 16, n_Y = 16, join 64                                              -> d_Z [2,1]: 64
#   re-partitions of the 8 x 4 tensor T (n = 32):
#     [1,2] or [2,1] -> [1,1]: n_p = 16, n_c = 32, n_int = 16: (2-1)*1*(32+16) = 48
#     [1,1] -> [1,2] or [2,1]: n_p = 32, n_c = 16, n_int = 16: first term 0, n_p != n_int: + 32*2 = 64
#     [1,2] <-> [2,1]:         n_p = n_c = 16, n_int = 8: (2-1)*2*32 = 64, + 16*2 = 32: 96
#   U (one input, pays p n_X = 2*16 = 32 under either cut):
#     k cut, wants T as [1,2]: min(80+0, 80+64, 64+96) = 80   -> d_Z [1,2]: 112, T arrives as [1,2]
#     i cut, wants T as [2,1]: min(80+96, 80+64, 64+0) = 64   -> d_Z [2,1]:  96, T arrives as [2,1]
#   S (i=8, k=4, l=16; V lies off the path and costs nothing):
#     l cut: join 2*(32+64) = 192, U wanted as [1,1]: min(112+48, 96+48) = 144              -> d_Z [1,2]: 336
#     k cut: join 2*(16+128) = 288, U wanted as [1,2]: min(112, 96+96) = 112                -> d_Z [2,1]: 400
#     i cut: join 2*(16+64) = 160, n_agg = 2, n_Z = 64, agg 64, U wanted as [2,1]: 96       -> d_Z [1,1]: 320
#   so the first path T, U, S ends at 320 and is labelled i, i, i.  V alone (T off the path, free):
#     l cut: 2*(32+32) = 128;  k cut: 2*(16+32) = 96 + agg 128 = 224;  i cut: 2*(16+64) = 160  -> l cut.
#   With every edge counted: T 64, U 32, V 128 + 48 (T from [2,1] to [1,1]), S 160 + 64 + 384 (V from [1,2] to
#   [2,1] on its 8 x 16 tensor: n_p = n_c = 64, n_int = 32, n = 128: (2-1)*2*128 = 256, + 64*2 = 128) = 880.
#   Cutting all four vertices along i costs 64 + 32 + 160 + 224 = 480: the edges between paths are what the
#   heuristic does not see.
def test_path_decomposition_of_a_graph_worked_by_hand():
    vs = shared_result_graph()
    g = {v.name: v for v in vs}
    # two chains of three vertices tie; the one through the vertex created first wins, V is left for a path of its own
    assert P.longest_path(vs, ["T", "U", "V", "S"]) == ["T", "U", "S"]
    assert P.longest_path(vs, ["V"]) == ["V"]
    path = ["T", "U", "S"]
    M = P.dp_chain(g, [g[n] for n in path], set(zip(path[:-1], path[1:])), 2)
    costs = lambda name: {k: int(c) for k, (c, _, _) in M[name].items()}
    assert costs("T") == {(1, 2): 80, (1, 1): 80, (2, 1): 64}
    assert costs("U") == {(1, 2): 112, (2, 1): 96}
    assert costs("S") == {(1, 2): 336, (2, 1): 400, (1, 1): 320}
    assert M["U"][(1, 2)][2] == {"T": (1, 2)} and M["U"][(2, 1)][2] == {"T": (2, 1)}
    assert M["S"][(1, 2)][2] == {"U": (2, 1)} and M["S"][(2, 1)][2] == {"U": (1, 2)} and M["S"][(1, 1)][2] == {"U": (2, 1)}
    MV = P.dp_chain(g, [g["V"]], set(), 2)
    assert {k: int(c) for k, (c, _, _) in MV["V"].items()} == {(1, 2): 128, (1, 1): 224, (2, 1): 160}
    labels = P.eindecomp_paths(vs, 2)
    assert labels == {"T": {"i": 2, "j": 1, "k": 1}, "U": {"i": 2, "k": 1}, "S": {"i": 2, "k": 1, "l": 1}, "V": {"i": 1, "k": 1, "l": 2}}
    assert P.labelling_cost(vs, labels) == 880
    all_i = {"T": {"i": 2, "j": 1, "k": 1}, "U": {"i": 2, "k": 1}, "S": {"i": 2, "k": 1, "l": 1}, "V": {"i": 2, "k": 1, "l": 1}}
    assert P.labelling_cost(vs, all_i) == 480
    assert P.brute_force(vs, 2)[0] <= 480


def test_repartition_costs_used_in_the_worked_example():
    assert P.cost_repart([1, 1], [1, 2], [8, 4]) == 48 and P.cost_repart([1, 1], [2, 1], [8, 4]) == 48
    assert P.cost_repart([1, 2], [1, 1], [8, 4]) == 64 and P.cost_repart([2, 1], [1, 1], [8, 4]) == 64
    assert P.cost_repart([1, 2], [2, 1], [8, 4]) == 96 and P.cost_repart([2, 1], [1, 2], [8, 4]) == 96
    assert P.cost_repart([2, 1], [1, 2], [8, 16]) == 384
