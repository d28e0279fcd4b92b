"""GPU parity on randomly drawn EinSum graphs: a few inputs, three to six vertices that consume inputs and
earlier results (some results feed several vertices), a different random partitioning vector on every
vertex (so consecutive vertices disagree about how a tensor is cut), mixed dtypes.  What this reaches that
single-vertex cases cannot: repartition between producer and consumer, the workspace layout and its reuse
of dead intermediates, chains that look a little like a softmax without being one, and the planner's own
labelling of an arbitrary graph.  Every output is compared with the CPU oracle element by element."""
import os

import numpy as np
import pytest

from tests._parity import magnitudes, rtol_for, violations
from oracle.graph_ref import make_inputs, run_graph
from synth_inputs.workloads import Vertex, Workload

pytestmark = pytest.mark.gpu

N_GRAPHS = int(os.environ.get("EINDECOMP_RANDOM_GRAPHS", "40"))   # more graphs on request, same generator
BOUNDS = [4, 6, 8, 16, 24, 40]
# scalar functions that stay continuous in their arguments: a step function of a rounded intermediate may
# legitimately flip between two correct evaluations
MAP2 = ["mul", "add", "sub", "sqdiff", "absdiff", "silu_mul"]
MAP1 = ["ident", "scale", "relu"]
RED2 = [("mul", "sum")] * 4 + [("sqdiff", "sum"), ("absdiff", "max"), ("add", "max")]
RED1 = [("ident", "sum"), ("ident", "max"), ("relu", "sum"), ("scale", "max")]


def _divisors(n, cap):
    return [d for d in range(1, min(n, cap) + 1) if n % d == 0]


def draw_graph(seed):
    rng = np.random.default_rng(9_2410_02682 + seed)
    tensors = []                                      # (name, bound)
    vertices = []
    for i in range(int(rng.integers(2, 4))):
        rank = int(rng.integers(1, 4))
        bound = tuple(int(rng.choice(BOUNDS)) for _ in range(rank))
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        dist = {"dist": "uniform"} if rng.random() < 0.7 else {"dist": "normal", "std": 0.5}
        vertices.append(Vertex(f"I{i}", dtype, bound=bound, recipe=dist))
        tensors.append((f"I{i}", bound))
    parts = {"a": {}, "b": {}, "whole": {}}
    consumed = set()
    n_einsum = int(rng.integers(3, 7))
    for vi in range(n_einsum):
        letters = list("abcdefghij")
        rng.shuffle(letters)
        # favour recent results, so chains form; a result without labels (a scalar) is an output only
        usable = [j for j, (_, b) in enumerate(tensors) if len(b) > 0]
        weights = np.array([j + 1 for j in usable], dtype=np.float64)
        xi = int(rng.choice(usable, p=weights / weights.sum()))
        xname, xb = tensors[xi]
        lx = [letters.pop() for _ in xb]
        bound = dict(zip(lx, xb))
        binary = len(usable) > 1 and rng.random() < 0.7
        ly = None
        yname = None
        if binary:
            yi = int(rng.choice([j for j in usable if j != xi]))
            yname, yb = tensors[yi]
            ly = []
            for b in yb:
                cands = [l for l in lx if bound[l] == b and l not in ly]
                if cands and rng.random() < 0.65:
                    ly.append(str(rng.choice(cands)))
                else:
                    l = letters.pop()
                    bound[l] = b
                    ly.append(l)
        labels = list(dict.fromkeys(lx + (ly or [])))
        lz = [l for l in labels if rng.random() < 0.65]
        size = int(np.prod([bound[l] for l in lz])) if lz else 1
        while size > 60000:                           # keep results small enough to feed further vertices cheaply
            lz.pop()
            size = int(np.prod([bound[l] for l in lz])) if lz else 1
        rng.shuffle(lz)
        has_agg = len(lz) < len(labels)
        if binary:
            otimes, oplus = RED2[int(rng.integers(len(RED2)))] if has_agg else (MAP2[int(rng.integers(len(MAP2)))], "none")
        else:
            otimes, oplus = RED1[int(rng.integers(len(RED1)))] if has_agg else (MAP1[int(rng.integers(len(MAP1)))], "none")
        alpha = float(rng.choice([1.0, 0.5, -1.5])) if otimes in ("scale", "add") else 1.0
        spec = "".join(lx) + ("," + "".join(ly) if ly is not None else "") + "->" + "".join(lz)
        dtype = "bf16" if rng.random() < 0.4 else "f32"
        name = f"V{vi}"
        vertices.append(Vertex(name, dtype, spec=spec, otimes=otimes, oplus=oplus, alpha=alpha,
                               inputs=(xname,) if yname is None else (xname, yname)))
        consumed.add(xname)
        if yname is not None:
            consumed.add(yname)
        tensors.append((name, tuple(bound[l] for l in lz)))
        for pname in ("a", "b"):
            d, p = {}, 1
            for l in labels:
                k = int(rng.choice(_divisors(bound[l], 4)))
                if p * k <= 16:
                    d[l] = k
                    p *= k
            parts[pname][name] = d
    names = [v.name for v in vertices if not v.is_input]
    outputs = [n for n in names if n not in consumed]
    for n in names:
        if n not in outputs and rng.random() < 0.3:
            outputs.append(n)
    return Workload(f"random{seed}", 77_000 + seed, vertices, outputs, parts)


def draw_matrix_graph(seed):
    """Matrices with extents the matrix-core kernels accept, multiplied in random orders and layouts, with the odd
    element-wise vertex in between; every label may be cut, so partial slabs, their aggregation and a repartition
    between any two vertices are the rule."""
    rng = np.random.default_rng(5_2410_02682 + seed)
    ext = [64, 72, 136, 264]
    dims = [int(rng.choice(ext)) for _ in range(3)]               # few distinct extents, so operands fit together
    tensors, vertices = [], []
    for i in range(int(rng.integers(2, 5))):
        bound = (int(rng.choice(dims)), int(rng.choice(dims)))
        vertices.append(Vertex(f"I{i}", "bf16" if rng.random() < 0.8 else "f32", bound=bound,
                               recipe={"dist": "normal", "std": 0.25}))
        tensors.append((f"I{i}", bound))
    parts = {"a": {}, "b": {}, "whole": {}}
    consumed = set()
    for vi in range(int(rng.integers(3, 7))):
        weights = np.arange(1, len(tensors) + 1, dtype=np.float64)
        xi = int(rng.choice(len(tensors), p=weights / weights.sum()))
        yi = int(rng.choice([j for j in range(len(tensors)) if j != xi]))
        (xname, xb), (yname, yb) = tensors[xi], tensors[yi]
        pairs = [(a, b) for a in range(2) for b in range(2) if xb[a] == yb[b]]
        if xb == yb and rng.random() < 0.35:
            spec, otimes, oplus = "ij,ij->ij", str(rng.choice(["add", "sub", "mul", "silu_mul"])), "none"
            bound = {"i": xb[0], "j": xb[1]}
        elif pairs:
            a, b = pairs[int(rng.integers(len(pairs)))]
            lx = ["m", "m"]; lx[a] = "k"
            ly = ["n", "n"]; ly[b] = "k"
            lz = ["m", "n"] if rng.random() < 0.7 else ["n", "m"]
            spec, otimes, oplus = "".join(lx) + "," + "".join(ly) + "->" + "".join(lz), "mul", "sum"
            bound = {"m": xb[1 - a], "k": xb[a], "n": yb[1 - b]}
        else:
            spec, otimes, oplus = "ij->ji", "scale", "none"
            yname = None
            bound = {"i": xb[0], "j": xb[1]}
        lz = spec.split("->")[1]
        name = f"V{vi}"
        scale = 1.0 / 16 if oplus == "sum" else (0.5 if otimes == "scale" else 1.0)   # keeps products of products in range
        vertices.append(Vertex(name, "bf16" if rng.random() < 0.6 else "f32", spec=spec, otimes=otimes, oplus=oplus,
                               alpha=scale, inputs=(xname,) if yname is None else (xname, yname)))
        consumed.add(xname)
        if yname is not None:
            consumed.add(yname)
        tensors.append((name, tuple(bound[l] for l in lz)))
        for pname in ("a", "b"):
            d = {}
            for l, b in bound.items():
                d[l] = int(rng.choice([k for k in (1, 2, 4, 8) if b % (8 * k) == 0]))
            parts[pname][name] = d
    names = [v.name for v in vertices if not v.is_input]
    outputs = [n for n in names if n not in consumed]
    for n in names:
        if n not in outputs and rng.random() < 0.3:
            outputs.append(n)
    return Workload(f"matrices{seed}", 78_000 + seed, vertices, outputs, parts)


def _run(w, pname, inputs, merged=False):
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    r = GraphRunner(w, pname)
    try:
        if merged:
            E.tr_set_fused_aggregation(r.g, True)     # the alternative method: no partial slabs, no aggregation stage
        r.bind({k: to_device(t) for k, t in inputs.items()})
        r.run()
        torch.cuda.synchronize()
        return {n: to_host(r.output(n)) for n in r.out_names}
    finally:
        r.close()


@pytest.mark.parametrize("family,seed", [(f, s) for f in ("labels", "matrices") for s in range(N_GRAPHS)])
def test_random_graph_matches_oracle_under_every_labelling(family, seed):
    w = draw_graph(seed) if family == "labels" else draw_matrix_graph(seed)
    desc = "; ".join(f"{v.name}={v.spec}[{v.otimes}/{v.oplus}]({','.join(v.inputs)})" for v in w.einsum_vertices())
    print(f"graph {seed}: {desc}; outputs {w.outputs}", flush=True)
    inputs = make_inputs(w)
    ref = run_graph(w, inputs)
    mag = magnitudes(w, inputs)                       # what cancelling sums are held against (graph 1028 of the first family)
    rep = {}
    for pname, merged in (("a", False), ("b", False), ("whole", False), ("eindecomp:4", False), ("a", True), ("b", True)):
        got = _run(w, pname, inputs, merged)
        for name in w.outputs:
            r = ref[name].as_f64()
            assert got[name].shape == ref[name].shape
            bad, worst = violations(got[name].as_f64(), r, rtol_for(w, name), mag[name].as_f64(), report=rep)
            assert bad == 0, f"labelling {pname}{' (aggregation merged)' if merged else ''} output {name}: {bad} elements out of tolerance (worst {worst:.2f}x)"
    # The allowance for cancelling sums is there for sums that cancel to a millionth of their terms; a graph whose
    # outputs lean on it in more than a handful of elements has another problem.
    print(f"graph {seed}: {rep['leaned_on_magnitude']} elements needed the allowance for cancelling sums; "
          f"worst plain relative error on elements above the rms {rep['strict_worst']:.2e}", flush=True)
    n_out = sum(int(np.prod(ref[name].shape)) for name in w.outputs) * 6
    assert rep["leaned_on_magnitude"] <= max(8, n_out // 100), rep
