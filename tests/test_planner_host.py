"""The library's planner (host code, no GPU needed) against the planner oracle: costs and enumeration entry by entry,
the chosen labelling by its cost (several labellings can tie) and by validity."""
import math

import pytest

import paper_2410_02682_amd as E
from oracle import planner_ref as P
from synth_inputs import build_config
from tests.test_planner_oracle import chain, tree, diamond, shared_result_graph


def build(vs):
    g = E.einsum_graph_create()
    vid = {}
    for v in vs:
        if v.spec is None:
            vid[v.name] = E.einsum_graph_add_input(g, v.bound, "bf16")
        else:
            vid[v.name] = E.einsum_graph_add_einsum(g, v.spec, "mul" if len(v.inputs) == 2 else "ident", "sum", 1.0, [vid[n] for n in v.inputs], "bf16")
    return g, vid


def schema(vs, v):
    return P.unique_labels(P.split_spec(v.spec)[0])


def labels_of(g, vid, vs):
    out = {}
    for v in vs:
        if v.spec is not None:
            pl = E.einsum_graph_plan(g, vid[v.name])
            out[v.name] = dict(zip(pl["labels"], pl["d"]))
    return out


def test_costs_match_the_oracle_on_every_viable_vector():
    vs = chain(3, [16, 4, 32, 8], unary_tail=True)
    g, vid = build(vs)
    gd = {v.name: v for v in vs}
    for v in vs:
        if v.spec is None:
            continue
        b = P.label_bounds(gd, v)
        lab = schema(vs, v)
        for p in (1, 2, 8, 32):
            want = P.viable(v.spec, b, p)
            got = E.eindecomp_viable(g, vid[v.name], p)
            assert got == [[d[l] for l in lab] for d in want]          # same vectors in the same order
            for d in want:
                dv = [d[l] for l in lab]
                assert E.eg_cost_join(g, vid[v.name], dv) == P.cost_join(v.spec, b, d)
                assert E.eg_cost_agg(g, vid[v.name], dv) == P.cost_agg(v.spec, b, d)
    E.einsum_graph_destroy(g)


def test_repartition_cost_matches_the_oracle_and_the_printed_320():
    assert E.eg_cost_repart([8, 8], [4, 1], [2, 4]) == 320
    cuts = [1, 2, 4, 8]
    for bound in ([8, 8], [16, 8], [8, 24, 16]):
        for dc in __import__("itertools").product(cuts, repeat=len(bound)):
            for dp in __import__("itertools").product(cuts, repeat=len(bound)):
                assert E.eg_cost_repart(bound, dc, dp) == P.cost_repart(dc, dp, bound)
    with pytest.raises(E.EgError):
        E.eg_cost_repart([8, 8], [3, 1], [2, 4])                       # 3 does not divide 8
    # cuts that do not nest (blocks of 3 against blocks of 4) still have a value under the formula
    assert E.eg_cost_repart([12], [4], [3]) == P.cost_repart([4], [3], [12]) == 16


@pytest.mark.parametrize("vs,p", [(chain(3, [8, 8, 8, 8]), 4), (chain(3, [16, 4, 32, 8]), 8), (chain(4, [8, 16, 4, 8, 8]), 4),
                                  (chain(3, [8, 8, 8, 8], unary_tail=True), 4), (tree(), 4), (chain(5, [64, 256, 32, 512, 64, 128]), 16)])
def test_plan_is_the_optimum_on_graphs_without_shared_results(vs, p):
    g, vid = build(vs)
    cost, exact = E.eindecomp_plan(g, p)
    want, want_labels = P.eindecomp_tree(vs, p)
    assert exact and cost == want
    got = labels_of(g, vid, vs)
    assert P.labelling_cost(vs, got) == cost                            # the labelling set on the graph costs what was reported
    assert got == want_labels                                           # same tie-breaking, so even the vectors agree
    parts = E.eindecomp_labelling_cost(g)
    assert parts["total"] == cost
    E.einsum_graph_destroy(g)


def test_plan_on_a_graph_with_a_shared_result_follows_the_path_decomposition():
    vs = diamond()
    g, vid = build(vs)
    cost, exact = E.eindecomp_plan(g, 4)
    assert not exact
    got = labels_of(g, vid, vs)
    assert got == P.eindecomp_paths(vs, 4)
    assert cost == P.labelling_cost(vs, got) >= P.brute_force(vs, 4)[0]
    E.einsum_graph_destroy(g)


def test_plan_reproduces_the_path_decomposition_worked_by_hand():
    # the literals derived by hand in tests/test_planner_oracle.py (Section 8.4 with the costs of Section 7, p = 2)
    vs = shared_result_graph()
    g, vid = build(vs)
    cost, exact = E.eindecomp_plan(g, 2)
    assert not exact and cost == 880
    assert labels_of(g, vid, vs) == {"T": {"i": 2, "j": 1, "k": 1}, "U": {"i": 2, "k": 1}, "S": {"i": 2, "k": 1, "l": 1},
                                     "V": {"i": 1, "k": 1, "l": 2}}
    parts = E.eindecomp_labelling_cost(g)
    assert parts == dict(join=64 + 32 + 128 + 160, agg=64, repart=48 + 384, total=880)
    for name, d in (("T", [2, 1, 1]), ("U", [2, 1]), ("S", [2, 1, 1]), ("V", [2, 1, 1])):
        E.einsum_graph_set_partition(g, vid[name], d)
    assert E.eindecomp_labelling_cost(g)["total"] == 480
    E.einsum_graph_destroy(g)


@pytest.mark.parametrize("n", [2, 3, 4, 5])
def test_plan_labels_the_workload_graphs(n):
    w = build_config(n)
    vs = P.from_workload(w)
    g, vid = build(vs)
    cost, exact = E.eindecomp_plan(g, 8)
    got = labels_of(g, vid, vs)
    shared = any(len(c) > 1 for name, c in P.consumers_of(vs).items() if {v.name: v for v in vs}[name].spec is not None)
    assert exact == (not shared)
    want = P.eindecomp_paths(vs, 8) if shared else P.eindecomp_tree(vs, 8)[1]
    assert got == want and cost == P.labelling_cost(vs, got)
    for v in vs:
        if v.spec is not None:
            assert math.prod(got[v.name].values()) <= 8
    E.einsum_graph_destroy(g)


def test_plan_rejects_bad_arguments():
    vs = chain(2, [8, 8, 8])
    g, vid = build(vs)
    with pytest.raises(E.EgError):
        E.eindecomp_plan(g, 6)
    with pytest.raises(E.EgError):
        E.eindecomp_viable(g, vid["A0"], 4)                            # an input vertex
    with pytest.raises(E.EgError):
        E.eg_cost_join(g, vid["M1"], [3, 1, 1])                        # 3 does not divide 8
    E.einsum_graph_destroy(g)
