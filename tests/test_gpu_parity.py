"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.

Sizes are those the oracle finishes in seconds while every block still spans several kernel
tiles with ragged tails.  Full-size checks live in test_gpu_fullsize.py."""
import itertools
import math

import numpy as np
import pytest

from tests._parity import RTOL_BF16, RTOL_F32, rtol_for, single_vertex, tile_of, violations
from oracle.einsum_ref import einsum_ref
from oracle.graph_ref import make_inputs, run_graph, to_storage
from synth_inputs import build_config
from synth_inputs.prng import HostTensor, make_tensor, small_ints, uniform_pm1, normal

pytestmark = pytest.mark.gpu


def _gpu():
    import torch
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    return torch, GraphRunner, to_device, to_host


def _run(w, pname, inputs, outputs=None, contract=None):
    torch, GraphRunner, to_device, to_host = _gpu()
    r = GraphRunner(w, pname, outputs=outputs, contract=contract)
    try:
        r.bind({k: to_device(t) for k, t in inputs.items()})
        r.run()
        torch.cuda.synchronize()
        return {n: to_host(r.output(n)) for n in r.out_names}
    finally:
        r.close()


# ------------------------------------------------------------------ the five configurations, scaled down
CASES = [(n, p) for n in range(1, 8) for p in build_config(n, small=True).partitionings]
_ref_cache = {}


def _reference(n):
    if n not in _ref_cache:
        w = build_config(n, small=True)
        inp = make_inputs(w)
        _ref_cache[n] = (w, inp, run_graph(w, inp))
    return _ref_cache[n]


@pytest.mark.parametrize("n,pname", CASES)
def test_config_every_vertex_matches_oracle(n, pname):
    w, inp, ref = _reference(n)
    names = [v.name for v in w.einsum_vertices()]
    print(f"config {n} partitioning {pname}: all vertices as outputs", flush=True)
    got = _run(w, pname, inp, outputs=names)
    strict = {}
    for name in names:
        rep = {}
        bad, worst = violations(got[name].as_f64(), ref[name].as_f64(), rtol_for(w, name), report=rep)
        assert bad == 0, f"config {n} {pname} vertex {name}: {bad} elements out of tolerance (worst {worst:.2f}x)"
        strict[name] = rep["strict_worst"] / rtol_for(w, name)
        # on elements that are not small against the tensor the stated relative bound holds without the rms term
        assert rep["strict_worst"] <= rtol_for(w, name), f"config {n} {pname} vertex {name}: plain relative error {rep['strict_worst']:.2e}"
    worst_name = max(strict, key=strict.get)
    print(f"config {n} {pname}: worst plain relative error on elements above the rms: {strict[worst_name]:.3f} of the bound ({worst_name})", flush=True)


@pytest.mark.parametrize("tile", ["", "256x128", "256"])
@pytest.mark.parametrize("n,pname", CASES)
def test_config_outputs_through_workspace_match_oracle(n, pname, tile):
    # at these sizes the bf16 contraction kernel would always pick its small tile: the other passes force the larger ones
    w, inp, ref = _reference(n)
    print(f"config {n} partitioning {pname}: intermediates in the workspace, tile {tile or 'default'}", flush=True)
    got = _run(w, pname, inp, contract=dict(tile=tile_of(tile)) if tile else None)
    for name in w.outputs:
        bad, worst = violations(got[name].as_f64(), ref[name].as_f64(), rtol_for(w, name))
        assert bad == 0, f"config {n} {pname} output {name}: {bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("n,p", [(n, p) for n in range(1, 8) for p in (4, 16)])
def test_config_under_the_planners_own_labelling_matches_oracle(n, p):
    # the partitioning vectors chosen by eindecomp_plan instead of hand-written ones; the result may not depend on them
    w, inp, ref = _reference(n)
    print(f"config {n} labelled by the planner for p = {p}", flush=True)
    got = _run(w, f"eindecomp:{p}", inp)
    for name in w.outputs:
        bad, worst = violations(got[name].as_f64(), ref[name].as_f64(), rtol_for(w, name))
        assert bad == 0, f"config {n} planner p={p} output {name}: {bad} elements out of tolerance (worst {worst:.2f}x)"


# ------------------------------------------------------------------ contraction layouts, tails, label groups
LAYOUTS = [
    # spec, bound X, bound Y: K-contiguous / M-contiguous A x K-contiguous / N-contiguous B, ragged tails
    ("ij,jk->ik", (200, 328), (328, 136)),       # A k-contig, B n-contig
    ("ij,kj->ik", (200, 328), (136, 328)),       # A k-contig, B k-contig
    ("ji,jk->ik", (328, 200), (328, 136)),       # A m-contig, B n-contig
    ("ji,kj->ik", (328, 200), (136, 328)),       # A m-contig, B k-contig
    ("ij,jk->ki", (200, 328), (328, 136)),       # transposed output
    ("bshd,bthd->bhst", (2, 72, 3, 40), (2, 56, 3, 40)),
    ("bhst,bthd->bshd", (2, 3, 72, 56), (2, 56, 3, 40)),
    ("bshd,ahd->bsa", (2, 72, 3, 40), (88, 3, 40)),
    ("ijk,kl->ijl", (3, 40, 264), (264, 72)),
    ("bf,bh->fh", (264, 136), (264, 72)),
    ("ji,jk->ik", (100, 200), (100, 136)),       # K tail that is no multiple of 8 (both operands strided along K)
    ("ij,kj->ik", (200, 24), (136, 24)),         # K shorter than one stage
    ("ij,jk->ik", (264, 1384), (1384, 264)),     # many stages, odd count, tail of 40
    ("bshd,ahd->bsa", (2, 72, 3, 64), (88, 3, 64)),      # two contracted labels, every stage starts a new run of the inner one
    ("bshd,ahd->bsa", (2, 72, 3, 128), (88, 3, 128)),    # ... and runs of two stages
    ("bshd,ahd->bsa", (2, 72, 2, 192), (88, 2, 192)),    # ... runs of three: the stage pointers wrap at odd and even stages
    ("bshd,ahd->bsa", (2, 72, 3, 96), (88, 3, 96)),      # runs that are no whole number of stages: a full and a half-filled stage per run
    ("bshd,bthd->bhst", (2, 72, 3, 80), (2, 56, 3, 80)),  # ... as the single contracted label of a batched product
    ("bsha,had->bsd", (2, 72, 3, 40), (3, 40, 136)),     # ... with the second operand contiguous along its columns
]


@pytest.mark.parametrize("dtype,tile", [("bf16", "128"), ("bf16", "256x128"), ("bf16", "256"), ("f32", "128"), ("f32", "256"), ("f32", "")])
@pytest.mark.parametrize("spec,bx,by", LAYOUTS)
def test_contraction_layouts(spec, bx, by, dtype, tile):
    # the direct-to-LDS kernel has three tile shapes and would pick the small one (or, for fp32, the register-staged kernel)
    # for products this small: each is run; ("f32", "") is the library's own choice
    print(f"contraction {spec} {bx} {by} {dtype} tile {tile or 'default'}", flush=True)
    contract = dict(kernel="dma", tile=tile_of(tile)) if tile else None      # the direct-to-LDS kernel wherever the layout is eligible for it
    x = HostTensor.from_f32(uniform_pm1(11, 0, int(np.prod(bx))).reshape(bx), dtype)
    y = HostTensor.from_f32(uniform_pm1(11, 1, int(np.prod(by))).reshape(by), dtype)
    w = single_vertex(spec, x, y, "f32")
    ref = run_graph(w, {"X": x, "Y": y})["Z"]
    got = _run(w, "whole", {"X": x, "Y": y}, contract=contract)["Z"]
    bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_F32)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("spec,bx,by", [("ij,jk->ik", (4000, 72), (72, 2200)), ("ji,kj->ik", (100, 4000), (2200, 100))])
def test_fp32_contraction_with_many_tiles(spec, bx, by):
    # 16 x 9 tiles of 256 x 256 with ragged edges: enough of them for the fp32 kernel's eight-wave configuration
    print(f"fp32 contraction {spec} {bx} {by}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(21, 0, int(np.prod(bx))).reshape(bx), "f32")
    y = HostTensor.from_f32(uniform_pm1(21, 1, int(np.prod(by))).reshape(by), "f32")
    w = single_vertex(spec, x, y, "f32", parts={"whole": {}, "d": {"i": 2, "j": 2}})
    ref = run_graph(w, {"X": x, "Y": y})["Z"]
    for pname in ("whole", "d"):
        got = _run(w, pname, {"X": x, "Y": y})["Z"]
        bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_F32)
        assert bad == 0, f"{pname}: {bad} elements out of tolerance (worst {worst:.2f}x)"


def test_contraction_routes_to_mfma_and_bf16_output_rounds_once():
    torch, GraphRunner, to_device, to_host = _gpu()
    x = HostTensor.from_f32(normal(12, 0, 256 * 192, 1.0).reshape(256, 192), "bf16")
    y = HostTensor.from_f32(normal(12, 1, 192 * 128, 1.0).reshape(192, 128), "bf16")
    w = single_vertex("ij,jk->ik", x, y, "bf16", parts={"d": {"i": 2, "j": 2, "k": 2}})
    r = GraphRunner(w, "d")
    assert r.plan("Z")["kernel"] == "contract_mfma"
    r.close()
    ref = run_graph(w, {"X": x, "Y": y})["Z"]
    got = _run(w, "d", {"X": x, "Y": y})["Z"]
    bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_BF16)
    assert bad == 0
    # bf16 results differ from the oracle's by at most one bf16 ulp (a different tie), never more
    ulp = np.abs(ref.as_f64()) * 2.0 ** -7 + 1e-30
    assert np.all(np.abs(got.as_f64() - ref.as_f64()) <= ulp)


# ------------------------------------------------------------------ exact cases
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_integer_inputs_are_bit_identical_under_every_partitioning(dtype):
    # small-integer entries: every product and partial sum is exact in fp32, so every decomposition
    # (Section 4.3) must give the same bits as the undecomposed EinSum
    bx, by = (128, 256), (256, 64)
    x = HostTensor.from_f32(small_ints(13, 0, bx[0] * bx[1]).reshape(bx), dtype)
    y = HostTensor.from_f32(small_ints(13, 1, by[0] * by[1]).reshape(by), dtype)
    parts = {"d%d%d%d" % d: {"i": d[0], "j": d[1], "k": d[2]} for d in itertools.product([1, 2, 4, 8], repeat=3) if math.prod(d) in (1, 8, 64)}
    w = single_vertex("ij,jk->ik", x, y, "f32", parts=parts)
    ref = run_graph(w, {"X": x, "Y": y})["Z"].data
    for pname in parts:
        print(f"integer invariant {dtype} {pname}", flush=True)
        got = _run(w, pname, {"X": x, "Y": y})["Z"].data
        assert np.array_equal(got, ref), pname


def test_identity_and_all_ones_operands():
    eye = make_tensor({"dist": "identity"}, (256, 256), "bf16", 0, 0)
    x = HostTensor.from_f32(normal(14, 0, 128 * 256, 1.0).reshape(128, 256), "bf16")
    w = single_vertex("ij,jk->ik", x, eye, "bf16", parts={"d": {"i": 2, "j": 4, "k": 1}})
    got = _run(w, "d", {"X": x, "Y": eye})["Z"]
    assert np.array_equal(got.data, x.data)                       # X.I = X, bit for bit
    ones_a = make_tensor({"dist": "ones"}, (64, 8192), "bf16", 0, 0)
    ones_b = make_tensor({"dist": "ones"}, (8192, 64), "bf16", 0, 0)
    w = single_vertex("ij,jk->ik", ones_a, ones_b, "bf16", parts={"d": {"j": 16}})
    got = _run(w, "d", {"X": ones_a, "Y": ones_b})["Z"]
    assert np.all(got.as_f32() == 8192.0)


def test_two_runs_are_bit_identical():
    w, inp, _ = _reference(2)
    a = _run(w, "mix", inp)["ABC"].data
    b = _run(w, "mix", inp)["ABC"].data
    assert np.array_equal(a, b)


# ------------------------------------------------------------------ maps, reductions, extended operators
UNARY = ["ident", "scale", "relu", "exp", "log"]
BINARY = ["mul", "add", "sub", "div", "sqdiff", "absdiff", "exp_sub", "relu_grad", "silu_mul"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,part", [((96, 200), {"i": 2, "j": 4}), ((7, 13), {}), ((4, 6, 40), {"k": 5}),
                                        ((4099, 37), {}), ((3, 5), {})])      # dense, not cut, no multiple of 8: vectors and a partial last one
def test_every_scalar_function_elementwise(shape, part, dtype):
    labs = "ijk"[:len(shape)]
    n = int(np.prod(shape))
    x = HostTensor.from_f32((uniform_pm1(15, 0, n) * 3).reshape(shape), dtype)
    y = HostTensor.from_f32((uniform_pm1(15, 1, n) * 3).reshape(shape), dtype)
    xp = HostTensor.from_f32((np.abs(uniform_pm1(15, 2, n)) + 0.5).reshape(shape), dtype)
    rtol = RTOL_F32 if dtype == "f32" else RTOL_BF16
    for op in UNARY:
        src = xp if op == "log" else x
        w = single_vertex(f"{labs}->{labs}", src, None, dtype, otimes=op, oplus="none", alpha=0.75, parts={"p": part})
        ref = run_graph(w, {"X": src})["Z"]
        got = _run(w, "p", {"X": src})["Z"]
        bad, worst = violations(got.as_f64(), ref.as_f64(), rtol)
        assert bad == 0, (op, bad, worst)
    for op in BINARY:
        rhs = xp if op == "div" else y
        w = single_vertex(f"{labs},{labs}->{labs}", x, rhs, dtype, otimes=op, oplus="none", alpha=0.75, parts={"p": part})
        ref = run_graph(w, {"X": x, "Y": rhs})["Z"]
        got = _run(w, "p", {"X": x, "Y": rhs})["Z"]
        bad, worst = violations(got.as_f64(), ref.as_f64(), rtol)
        assert bad == 0, (op, bad, worst)


@pytest.mark.parametrize("spec,bx,by,otimes,oplus,part", [
    ("ij,i->ij", (64, 136), (64,), "exp_sub", "none", {"i": 2, "j": 1}),
    ("ij,j->ij", (64, 136), (136,), "add", "none", {"j": 17}),
    ("bhst,st->bhst", (2, 3, 40, 48), (40, 48), "add", "none", {"h": 3, "t": 2}),
    ("ij,ij->ji", (40, 72), (40, 72), "sub", "none", {"i": 2}),
    ("ij->i", (96, 1000), None, "ident", "max", {"j": 8}),
    ("ij->i", (96, 1000), None, "ident", "sum", {"i": 2, "j": 4}),
    ("ij->j", (96, 1000), None, "ident", "sum", {"i": 4}),
    ("ij->", (96, 1000), None, "exp", "sum", {"i": 2, "j": 2}),
    ("bhst->bhs", (2, 3, 40, 256), None, "ident", "max", {"t": 4}),
    ("bc,bc->", (64, 256), (64, 256), "mul", "sum", {"b": 8}),
    ("ij,jk->ik", (40, 72), (72, 24), "sqdiff", "sum", {"i": 2, "j": 2, "k": 2}),
    ("ij,jk->ik", (40, 72), (72, 24), "absdiff", "max", {"i": 2, "j": 2, "k": 2}),
    ("ij,jk->ki", (40, 72), (72, 24), "sqdiff", "sum", {"i": 2, "j": 2}),      # result along an X-only label: operands change places
    ("ij,jk->ki", (264, 136), (136, 200), "absdiff", "max", {"k": 5}),
    ("ij,jk->ki", (264, 136), (136, 200), "sub", "sum", {}),                    # not symmetric: they stay
    ("ij,jk->ki", (264, 136), (136, 200), "add", "max", {"j": 2}),              # alpha * x + y is not symmetric either
    ("ij,j->i", (40, 1024), (1024,), "mul", "sum", {"j": 2}),
    ("ij,jk->ik", (37, 53), (53, 29), "mul", "sum", {}),          # nothing divides a vector: scalar paths
    ("ij->", (256, 1024), None, "exp", "sum", {}),                # one output, long reduction: split into pieces
    ("ij->", (3000, 4096), None, "ident", "sum", {}),             # ... into a thousand of them
    ("ij->", (256, 1024), None, "ident", "max", {"i": 2}),        # split pieces x two partial blocks
    ("bij,bij->b", (3, 200, 328), (3, 200, 328), "mul", "sum", {"i": 2}),
])
def test_maps_reductions_and_extended_operators(spec, bx, by, otimes, oplus, part):
    print(f"{spec} {otimes}/{oplus} {part}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(16, 0, int(np.prod(bx))).reshape(bx), "f32")
    y = None if by is None else HostTensor.from_f32(uniform_pm1(16, 1, int(np.prod(by))).reshape(by), "f32")
    w = single_vertex(spec, x, y, "f32", otimes=otimes, oplus=oplus, alpha=0.5, parts={"p": part})
    inputs = {"X": x} if y is None else {"X": x, "Y": y}
    ref = run_graph(w, inputs)["Z"]
    got = _run(w, "p", inputs)["Z"]
    bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_F32)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,n,otimes,oplus,part", [
    (1000, 8, "ident", "sum", {}), (1000, 24, "ident", "max", {}), (4099, 64, "ident", "sum", {}),          # 8 lanes per output
    (1237, 120, "ident", "sum", {}), (1237, 128, "relu", "sum", {"i": 1}),                                  # 16
    (2050, 136, "ident", "max", {}), (2048, 256, "ident", "sum", {"i": 4}),                                 # 32
    (1500, 264, "ident", "sum", {}), (1100, 512, "exp", "sum", {}), (1025, 504, "ident", "max", {"i": 5}),   # 64
    (1100, 520, "ident", "sum", {}),                                                                        # more than one vector per lane
    (1200, 512, "ident", "sum", {"j": 4}), (1200, 384, "ident", "max", {"j": 3, "i": 2}),                   # pieces of rows into partial slabs
    (4096, 96, "mul", "sum", {}), (4096, 96, "mul_bcast", "sum", {"i": 2}), (2052, 40, "sqdiff", "sum", {}),   # two operands
])
def test_row_reductions_over_short_rows(rows, n, otimes, oplus, part, dtype):
    """Rows short enough that several outputs share a wave (8 to 64 lanes per output, four outputs per lane group):
    every group size, output counts that fill neither the last group nor the last workgroup, rows that leave lanes
    idle, rows cut into partial slabs, a second operand of the same shape or one value per row."""
    print(f"{rows} x {n} {otimes}/{oplus} {part} {dtype}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(31, 0, rows * n).reshape(rows, n), dtype)
    spec, y = "ij->i", None
    if otimes in ("mul", "sqdiff"):
        spec, y = "ij,ij->i", HostTensor.from_f32(uniform_pm1(31, 1, rows * n).reshape(rows, n), dtype)
    elif otimes == "mul_bcast":
        spec, otimes, y = "ij,i->i", "mul", HostTensor.from_f32(uniform_pm1(31, 1, rows).reshape(rows), dtype)
    w = single_vertex(spec, x, y, "f32", otimes=otimes, oplus=oplus, parts={"p": part})
    inputs = {"X": x} if y is None else {"X": x, "Y": y}
    ref = run_graph(w, inputs)["Z"]
    got = _run(w, "p", inputs)["Z"]
    bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_F32)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("dtype,out_dtype", [("f32", "f32"), ("bf16", "f32"), ("bf16", "bf16")])
@pytest.mark.parametrize("spec,bx,by,otimes,oplus,part", [
    ("ij->j", (1000, 264), None, "ident", "sum", {}),                     # column sums: few outputs, pieces into slabs
    ("ij->j", (1000, 264), None, "ident", "max", {"i": 4}),               # the reduced label cut as well
    ("ij->j", (333, 4096), None, "relu", "sum", {"j": 4}),
    ("bij->bj", (5, 200, 136), None, "ident", "sum", {"b": 5}),           # the middle label goes
    ("bij->j", (5, 200, 136), None, "ident", "sum", {"i": 2}),            # two reduced labels that do not fuse with a cut between
    ("ibj->bj", (70, 3, 72), None, "exp", "sum", {}),
    ("ij,ij->j", (700, 200), (700, 200), "mul", "sum", {"i": 7}),
    ("ij,j->j", (700, 200), (200,), "sqdiff", "sum", {}),
    ("ij,i->j", (700, 200), (700,), "mul", "sum", {"j": 5}),              # one value of Y per reduction step
    ("i,ij->j", (700,), (700, 200), "mul", "sum", {"i": 2}),              # the matrix is the second operand
    ("bi,ij->bj", (3, 90), (90, 136), "absdiff", "max", {}),
    ("ij->j", (70000, 8), None, "ident", "sum", {}),                      # one vector of outputs, a long walk: 64 pieces
    ("ij->j", (20, 64), None, "ident", "sum", {}),
])
def test_reductions_over_leading_labels(spec, bx, by, otimes, oplus, part, dtype, out_dtype):
    """The outputs' innermost label is contiguous in X, the reduced labels lie in front of it: lanes own vectors of
    outputs and walk the reduction, which is cut into pieces when there are few outputs."""
    print(f"{spec} {bx} {otimes}/{oplus} {part} {dtype}->{out_dtype}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(41, 0, int(np.prod(bx))).reshape(bx), dtype)
    y = None if by is None else HostTensor.from_f32(uniform_pm1(41, 1, int(np.prod(by))).reshape(by), dtype)
    w = single_vertex(spec, x, y, out_dtype, otimes=otimes, oplus=oplus, parts={"p": part, "whole": {}})
    inputs = {"X": x} if y is None else {"X": x, "Y": y}
    ref = run_graph(w, inputs)["Z"]
    for pname in ("p", "whole"):
        import paper_2410_02682_amd as E
        from paper_2410_02682_amd.runner import GraphRunner
        r = GraphRunner(w, pname)
        kernel = r.plan("Z")["kernel"]
        r.close()
        assert kernel == "reduce_row", kernel
        got = _run(w, pname, inputs)["Z"]
        bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_BF16 if out_dtype == "bf16" else RTOL_F32)
        assert bad == 0, f"{pname}: {bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("dtype,out_dtype", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("spec,bx,by,otimes,part", [
    ("ij->ji", (200, 136), None, "ident", {}),                            # ragged 64 x 64 tiles in both directions
    ("ij->ji", (64, 64), None, "scale", {"i": 2, "j": 4}),
    ("ij->ji", (8, 1000), None, "relu", {"j": 5}),
    ("bij->bji", (3, 72, 264), None, "ident", {"b": 3}),
    ("bhst->bhts", (2, 3, 80, 136), None, "exp", {"h": 3, "s": 2}),
    ("ibj->jbi", (72, 5, 40), None, "ident", {}),                         # a label between the two that swap
    ("ij,ji->ij", (136, 200), (200, 136), "add", {"i": 2}),               # the second operand is the transposed one
    ("ij,ji->ji", (136, 200), (200, 136), "sub", {"j": 5}),               # the first one is
    ("ij,i->ji", (136, 200), (136,), "mul", {}),                          # transposed operand and one value per column
    ("bij,j->bji", (2, 72, 64), (64,), "sqdiff", {}),
])
def test_elementwise_vertices_with_a_transposed_operand(spec, bx, by, otimes, part, dtype, out_dtype):
    print(f"{spec} {bx} {otimes} {part} {dtype}->{out_dtype}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(51, 0, int(np.prod(bx))).reshape(bx), dtype)
    y = None if by is None else HostTensor.from_f32(uniform_pm1(51, 1, int(np.prod(by))).reshape(by), dtype)
    w = single_vertex(spec, x, y, out_dtype, otimes=otimes, oplus="none", alpha=-0.75, parts={"p": part, "whole": {}})
    inputs = {"X": x} if y is None else {"X": x, "Y": y}
    ref = run_graph(w, inputs)["Z"]
    for pname in ("p", "whole"):
        got = _run(w, pname, inputs)["Z"]
        bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_BF16 if out_dtype == "bf16" else RTOL_F32)
        assert bad == 0, f"{pname}: {bad} elements out of tolerance (worst {worst:.2f}x)"
        if otimes == "ident" and dtype == out_dtype:                    # a pure permutation moves bits
            assert np.array_equal(got.data, ref.data)


@pytest.mark.parametrize("dtype,out_dtype", [("bf16", "bf16"), ("f32", "f32")])
@pytest.mark.parametrize("spec,bx,by,otimes,oplus,part", [
    ("ij,jk->ik", (256, 8192), (8192, 128), "mul", "sum", {}),                # 2 tiles, long K: cut 8 ways by the executor
    ("ij,kj->ik", (136, 4096), (72, 4096), "mul", "sum", {"j": 2}),           # on top of the vertex's own cut
    ("ij,jk->ki", (64, 8192), (8192, 264), "mul", "sum", {"k": 3}),
    ("bij,bjk->bik", (3, 64, 4096), (3, 4096, 64), "mul", "sum", {"b": 3}),
    ("ij,jk->ik", (64, 4096), (4096, 64), "sqdiff", "sum", {}),
    ("ij,jk->ik", (64, 4096), (4096, 64), "absdiff", "max", {"i": 2}),
])
def test_underfilled_contractions_with_a_long_reduction(spec, bx, by, otimes, oplus, part, dtype, out_dtype):
    """Few output tiles and thousands of contracted elements: the executor cuts the contracted label further than the
    vertex's vector says and aggregates the extra partial slabs; the result is that of the vertex as given."""
    print(f"{spec} {bx} {by} {otimes}/{oplus} {part} {dtype}->{out_dtype}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(61, 0, int(np.prod(bx))).reshape(bx), dtype)
    y = HostTensor.from_f32(uniform_pm1(61, 1, int(np.prod(by))).reshape(by), dtype)
    w = single_vertex(spec, x, y, out_dtype, otimes=otimes, oplus=oplus, parts={"p": part})
    ref = run_graph(w, {"X": x, "Y": y})["Z"]
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    import torch
    r = GraphRunner(w, "p")
    try:
        r.bind({"X": to_device(x), "Y": to_device(y)})
        E.tr_profile_enable(r.g, 8)
        r.run()
        torch.cuda.synchronize()
        stages = [rec["stage"] for rec in E.tr_profile_read(r.g)]
        assert stages == ["join", "aggregate"], stages               # partial slabs even where the vertex's vector cuts no contracted label
        got = to_host(r.output("Z"))
    finally:
        r.close()
    bad, worst = violations(got.as_f64(), ref.as_f64(), RTOL_BF16 if out_dtype == "bf16" else RTOL_F32)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"


def test_softmax_pins_on_the_gpu():
    # constant rows of power-of-two length give exactly 1/n; rows sum to one; a row of 1000s needs the max subtraction
    from synth_inputs.workloads import Vertex, Workload
    rows = np.stack([np.full(64, 3.25), np.full(64, 1000.0), np.linspace(-4, 4, 64), -np.arange(64.0)]).astype(np.float32)
    x = HostTensor(rows, "f32")
    vs = [Vertex("X", "f32", bound=(4, 64)),
          Vertex("C", "f32", spec="ij->i", otimes="ident", oplus="max", inputs=("X",)),
          Vertex("E", "f32", spec="ij,i->ij", otimes="exp_sub", oplus="none", inputs=("X", "C")),
          Vertex("S", "f32", spec="ij->i", otimes="ident", oplus="sum", inputs=("E",)),
          Vertex("P", "f32", spec="ij,i->ij", otimes="div", oplus="none", inputs=("E", "S"))]
    for part in ({}, {"j": 4}, {"i": 2, "j": 8}):
        w = Workload("softmax", 0, vs, ["P"], {"p": {v.name: {l: d for l, d in part.items() if l in v.spec.split("->")[0]} for v in vs if not v.is_input}})
        P = _run(w, "p", {"X": x})["P"].as_f64()
        assert np.array_equal(P[0], np.full(64, 1 / 64))
        assert np.array_equal(P[1], np.full(64, 1 / 64))
        assert np.allclose(P.sum(axis=1), 1.0, atol=1e-6)
        ref = run_graph(w, {"X": x})["P"].as_f64()
        assert violations(P, ref, RTOL_F32)[0] == 0


# ------------------------------------------------------------------ tr_aggregate on its own
@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_tr_aggregate_sum_max_and_strided_output(out_dtype):
    torch, GraphRunner, to_device, to_host = _gpu()
    import paper_2410_02682_amd as E
    n_agg, shape = 8, (48, 136)
    slab = (np.round(uniform_pm1(17, 0, shape[0] * shape[1]) * 64) / 64).astype(np.float32).reshape(shape)   # short mantissas
    parts = torch.from_numpy(np.stack([slab] * n_agg)).cuda()
    tdt = torch.float32 if out_dtype == "f32" else torch.bfloat16
    out = torch.zeros(shape, dtype=tdt, device="cuda")
    rel = E.tensor_partition(out.data_ptr(), out_dtype, shape, [1, 1])
    E.tr_aggregate("sum", parts.data_ptr(), n_agg, slab.size, rel, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = to_storage(n_agg * slab.astype(np.float64), out_dtype) if out_dtype == "f32" else HostTensor.from_f32((n_agg * slab).astype(np.float32), "bf16")
    assert np.array_equal(to_host(out).data, want.data)            # eight copies: exactly 8x, then one rounding
    E.tensor_relation_destroy(rel)
    # max over different slabs, into a strided (transposed) destination
    rnd = uniform_pm1(17, 1, n_agg * slab.size).reshape((n_agg,) + shape)
    parts = torch.from_numpy(rnd).cuda()
    buf = torch.zeros((shape[1], shape[0]), dtype=tdt, device="cuda")
    rel = E.tensor_partition(buf.data_ptr(), out_dtype, shape, [1, 1], strides=[1, shape[0]])
    E.tr_aggregate("max", parts.data_ptr(), n_agg, slab.size, rel, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = HostTensor.from_f32(rnd.max(axis=0), out_dtype)
    assert np.array_equal(to_host(buf.t()).data, want.data)
    E.tensor_relation_destroy(rel)
    with pytest.raises(E.EgError):
        rel = E.tensor_partition(out.data_ptr(), out_dtype, shape, [1, 1])
        try:
            E.tr_aggregate("sum", parts.data_ptr(), n_agg, slab.size + 1, rel, 0)
        finally:
            E.tensor_relation_destroy(rel)


@pytest.mark.parametrize("n_agg,shape", [(100, (3,)), (512, (1,)), (33, (5, 7)), (300, (64, 64)), (40, (65, 64))])
def test_tr_aggregate_of_many_slabs_adds_in_ascending_order(n_agg, shape):
    # the reference is the plain loop in fp32, ((p0 + p1) + p2) + ...: every variant of the kernel (one lane per output,
    # one wave per output with 64 slabs fetched at a time) must reproduce it bit for bit
    torch, GraphRunner, to_device, to_host = _gpu()
    import paper_2410_02682_amd as E
    n = int(np.prod(shape))
    rnd = normal(19, n_agg, n_agg * n, 3.0).reshape(n_agg, n)
    parts = torch.from_numpy(rnd).cuda()
    for op in ("sum", "max"):
        out = torch.zeros(shape, dtype=torch.float32, device="cuda")
        rel = E.tensor_partition(out.data_ptr(), "f32", shape, [1] * len(shape))
        E.tr_aggregate(op, parts.data_ptr(), n_agg, n, rel, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        E.tensor_relation_destroy(rel)
        acc = rnd[0].copy()
        for a in range(1, n_agg):
            acc = (acc + rnd[a]).astype(np.float32) if op == "sum" else np.maximum(acc, rnd[a])
        assert np.array_equal(out.cpu().numpy().ravel(), acc), (op, n_agg, shape)


def test_strided_input_relation_and_small_workspace_is_rejected():
    torch, GraphRunner, to_device, to_host = _gpu()
    import paper_2410_02682_amd as E
    xt = HostTensor.from_f32(uniform_pm1(18, 0, 96 * 64).reshape(96, 64), "f32")     # stored as [j, i]
    y = HostTensor.from_f32(uniform_pm1(18, 1, 96 * 40).reshape(96, 40), "f32")
    g = E.einsum_graph_create()
    a = E.einsum_graph_add_input(g, [64, 96], "f32")
    b = E.einsum_graph_add_input(g, [96, 40], "f32")
    z = E.einsum_graph_add_einsum(g, "ij,jk->ik", "mul", "sum", 1.0, [a, b], "f32")
    E.einsum_graph_set_partition(g, z, [2, 2, 1])
    E.einsum_graph_mark_output(g, z)
    E.tr_set_fused_aggregation(g, False)                     # the two-stage path: partial slabs in the workspace
    dx, dy = to_device(xt), to_device(y)
    out = torch.empty((64, 40), dtype=torch.float32, device="cuda")
    ra = E.tensor_partition(dx.data_ptr(), "f32", [64, 96], [2, 2], strides=[1, 64])   # a transposed view
    rb = E.tensor_partition(dy.data_ptr(), "f32", [96, 40], [2, 1])
    rz = E.tensor_partition(out.data_ptr(), "f32", [64, 40], [2, 1])
    need = E.tr_workspace_bytes(g)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    with pytest.raises(E.EgError) as ei:
        E.tr_execute(g, [ra, rb], [rz], ws.data_ptr(), need - 256, torch.cuda.current_stream().cuda_stream)
    assert ei.value.code == -9
    E.tr_execute(g, [ra, rb], [rz], ws.data_ptr(), need, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ref = einsum_ref("ji,jk->ik", xt.data, y.data, out_dtype="f32")
    assert violations(to_host(out).as_f64(), ref, RTOL_F32)[0] == 0
    for r in (ra, rb, rz):
        E.tensor_relation_destroy(r)
    E.einsum_graph_destroy(g)


def test_profile_records_every_launch():
    torch, GraphRunner, to_device, to_host = _gpu()
    import paper_2410_02682_amd as E
    w, inp, _ = _reference(2)
    r = GraphRunner(w, "mix")
    r.bind({k: to_device(t) for k, t in inp.items()})
    E.tr_profile_enable(r.g, 16)
    r.run()
    torch.cuda.synchronize()
    rec = E.tr_profile_read(r.g)
    assert [(x["stage"], x["kernel"]) for x in rec] == [("join", "contract_mfma"), ("aggregate", "none")] * 2
    assert all(x["ms"] > 0 for x in rec)
    r.close()


# ------------------------------------------------------------------ fused softmax chains
def _softmax_workload(bound, dtype, with_add, stats_consumed, stat_dtype="f32"):
    from synth_inputs.workloads import Vertex, Workload
    labs = "bhst"[4 - len(bound):]
    row = labs[:-1]
    vs = [Vertex("T", dtype, bound=tuple(bound), recipe={"dist": "normal", "std": 2.0})]
    src = "T"
    if with_add:
        vs.append(Vertex("M", "f32", bound=tuple(bound[-2:]), recipe={"dist": "causal_mask"}))
        vs.append(Vertex("T2", dtype, spec=f"{labs},{labs[-2:]}->{labs}", otimes="add", oplus="none", alpha=0.25, inputs=("T", "M")))
        src = "T2"
    vs += [
        Vertex("C", stat_dtype, spec=f"{labs}->{row}", otimes="ident", oplus="max", inputs=(src,)),
        Vertex("E", dtype, spec=f"{labs},{row}->{labs}", otimes="exp_sub", oplus="none", inputs=(src, "C")),
        Vertex("S", stat_dtype, spec=f"{labs}->{row}", otimes="ident", oplus="sum", inputs=("E",)),
        Vertex("P", dtype, spec=f"{labs},{row}->{labs}", otimes="div", oplus="none", inputs=("E", "S")),
    ]
    outs = ["P"]
    if stats_consumed:
        vs.append(Vertex("logS", "f32", spec=f"{row}->{row}", otimes="log", oplus="none", inputs=("S",)))
        outs += ["logS", "C"]
    first = labs[0]
    parts = {"whole": {}, "rows2": {v.name: {first: 2} for v in vs if v.spec}}
    # every vertex of the chain cut differently (even along the softmax label, except at the division): the fused
    # pass runs under the division's vector alone
    second = labs[-2]
    mixed = {"C": {labs[-1]: 2}, "E": {second: 2, labs[-1]: 4}, "S": {first: 2, labs[-1]: 2}, "P": {second: 2}, "T2": {first: 2, second: 2}, "logS": {}}
    parts["mixed"] = {v.name: mixed[v.name] for v in vs if v.spec}
    return Workload("softmax_chain", 77, vs, outs, parts, {})


_SOFTMAX_CASES = [((6, 40, 2048), "bf16", True, False), ((2, 3, 24, 1024), "bf16", True, True),
                  ((50, 520), "f32", False, True), ((12, 100), "f32", False, False),
                  ((4, 12, 100), "bf16", True, True), ((4, 8192), "bf16", False, False),
                  # rows of a workgroup share the added row (4, 8 or 16 rows lack its labels)
                  ((4, 2, 16, 512), "bf16", True, False), ((8, 24, 2048), "bf16", True, True),
                  ((4, 8, 4096), "bf16", True, False), ((4, 16, 1024), "f32", True, True),
                  ((16, 8, 8192), "bf16", True, False),
                  # all-bf16 chains with whole groups of four rows per wave: no added operand, a shared row of it, its rows one by one
                  ((32, 1024), "bf16", False, True), ((16, 4, 32, 1024), "bf16", True, False), ((4, 4, 8, 2048), "bf16", True, True),
                  ((2, 6, 16, 256), "bf16", True, True)]
# ... and the bf16 chains with rows of up to 2048 elements once more with row maxima and row sums stored as bf16: the
# exponentials and the division then see them rounded, written or not
_SOFTMAX_CASES = [c + ("f32",) for c in _SOFTMAX_CASES] + [c + ("bf16",) for c in _SOFTMAX_CASES if c[1] == "bf16" and c[0][-1] <= 2048]


@pytest.mark.parametrize("bound,dtype,with_add,stats,stat_dtype", _SOFTMAX_CASES)
def test_fused_softmax_matches_oracle_and_the_separate_vertices(bound, dtype, with_add, stats, stat_dtype):
    torch, GraphRunner, to_device, to_host = _gpu()
    import paper_2410_02682_amd as E
    w = _softmax_workload(bound, dtype, with_add, stats, stat_dtype)
    inp = make_inputs(w)
    ref = run_graph(w, inp)
    for pname in ("whole", "rows2", "mixed"):
        print(f"softmax chain {bound} {dtype} add={with_add} stats={stats} statistics stored as {stat_dtype} {pname}", flush=True)
        res = {}
        for fuse in (True, False):
            r = GraphRunner(w, pname)
            try:
                E.tr_set_fusion(r.g, fuse)
                r.bind({k: to_device(t) for k, t in inp.items()})
                E.tr_profile_enable(r.g, 32)
                r.run()
                torch.cuda.synchronize()
                kinds = [x["kernel"] for x in E.tr_profile_read(r.g)]
                assert ("softmax_fused" in kinds) == fuse
                if fuse:
                    assert len(kinds) == 1       # the fused pass; the logarithm of the row sums, when there is one, is evaluated in it
                res[fuse] = {n: to_host(r.output(n)) for n in r.out_names}
            finally:
                r.close()
        for n in w.outputs:
            rt = rtol_for(w, n)
            bad, worst = violations(res[True][n].as_f64(), ref[n].as_f64(), rt)
            assert bad == 0, f"{n} fused: {bad} elements out of tolerance (worst {worst:.2f}x)"
            # against the separate vertices: the same roundings, only the order of the row sum differs
            a, b = res[True][n].as_f64(), res[False][n].as_f64()
            ulp = np.abs(b) * 2.0 ** -7 + 1e-30 if w.vertex(n).dtype == "bf16" else (np.abs(b) + 1.0) * 2.0 ** -20
            if n == "logS" and stat_dtype == "bf16":
                ulp = np.full_like(b, 2.0 ** -7)          # the logarithm of a row sum that may differ by one bf16 unit
            assert np.all(np.abs(a - b) <= ulp), f"{n}: fused and separate results differ by more than one unit in the last place"


# ------------------------------------------------------------------ the whole step inside a HIP graph
@pytest.mark.parametrize("n,pname", [(3, "mixed"), (3, "batch8"), (4, "heads8"), (5, "k16")])
def test_execute_can_be_captured_into_a_hip_graph_and_replayed(n, pname):
    # tr_execute only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
    # caller may capture it; every replay, with the program's own eager work in between, must give the eager result
    torch, GraphRunner, to_device, to_host = _gpu()
    w, inp, ref = _reference(n)
    print(f"config {n} {pname} captured into a graph", flush=True)
    r = GraphRunner(w, pname)
    try:
        r.bind({k: to_device(t) for k, t in inp.items()})
        r.run()
        torch.cuda.synchronize()
        eager = {name: r.output(name).clone() for name in r.out_names}
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                r.run(torch.cuda.current_stream())
        torch.cuda.synchronize()
        for rep in range(3):
            for name in r.out_names:
                r.output(name).zero_()
            r.workspace.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for name in r.out_names:
                assert torch.equal(r.output(name), eager[name]), f"replay {rep}: {name} differs from the eager result"
        del g
    finally:
        r.close()


def test_fused_softmax_with_transposed_input_and_output_relations():
    # the source arrives as a transposed view and the result goes into one: the pass cannot use 16-byte accesses
    # along its rows and takes the workgroup-per-row variant
    torch, GraphRunner, to_device, to_host = _gpu()
    import paper_2410_02682_amd as E
    s_, t_ = 48, 200
    xt = HostTensor.from_f32(normal(31, 0, s_ * t_, 2.0).reshape(t_, s_), "f32")         # stored as [t, s]
    g = E.einsum_graph_create()
    x = E.einsum_graph_add_input(g, [s_, t_], "f32")
    c = E.einsum_graph_add_einsum(g, "st->s", "ident", "max", 1.0, [x], "f32")
    e = E.einsum_graph_add_einsum(g, "st,s->st", "exp_sub", "none", 1.0, [x, c], "f32")
    sm = E.einsum_graph_add_einsum(g, "st->s", "ident", "sum", 1.0, [e], "f32")
    p = E.einsum_graph_add_einsum(g, "st,s->st", "div", "none", 1.0, [e, sm], "f32")
    for v in (c, e, sm, p):
        E.einsum_graph_set_partition(g, v, [2, 1])
    E.einsum_graph_mark_output(g, p)
    E.tr_set_fusion(g, True)
    dx = to_device(xt)
    out = torch.zeros((t_, s_), dtype=torch.float32, device="cuda")                         # P stored as [t, s] too
    rx = E.tensor_partition(dx.data_ptr(), "f32", [s_, t_], [2, 1], strides=[1, s_])
    rp = E.tensor_partition(out.data_ptr(), "f32", [s_, t_], [2, 1], strides=[1, s_])
    assert E.tr_workspace_bytes(g) == 0                                                     # fused: no intermediate exists
    E.tr_profile_enable(g, 8)
    E.tr_execute(g, [rx], [rp], 0, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert [k["kernel"] for k in E.tr_profile_read(g)] == ["softmax_fused"]
    x64 = xt.data.astype(np.float64).T                                                      # [s, t]
    ex = np.exp(x64 - x64.max(axis=1, keepdims=True))
    ref = ex / ex.sum(axis=1, keepdims=True)
    got = to_host(out).as_f64().T
    assert violations(got, ref, RTOL_F32)[0] == 0
    assert np.allclose(got.sum(axis=1), 1.0, atol=1e-5)
    for r in (rx, rp):
        E.tensor_relation_destroy(r)
    E.einsum_graph_destroy(g)


# ------------------------------------------------------------------ aggregation merged into the contraction kernel
@pytest.mark.parametrize("n,pname", [(1, "d222"), (2, "mix"), (2, "splitk8"), (3, "batch8"), (4, "heads8"), (5, "k16"), (6, "d222"), (7, "d222"), (7, "j8")])
def test_contractions_with_the_aggregation_merged_into_the_kernel_match_oracle(n, pname):
    torch, GraphRunner, to_device, to_host = _gpu()
    import paper_2410_02682_amd as E
    w, inp, ref = _reference(n)
    print(f"config {n} {pname}: aggregation inside the contraction kernels", flush=True)
    r = GraphRunner(w, pname)
    try:
        two_stage = E.tr_workspace_bytes(r.g)
        E.tr_set_fused_aggregation(r.g, True)
        merged_ws = E.tr_workspace_bytes(r.g)                   # the partial slabs of the contractions are gone
        assert merged_ws < two_stage if n in (2, 5) else merged_ws <= two_stage
        r.bind({k: to_device(t) for k, t in inp.items()})
        E.tr_profile_enable(r.g, 64)
        r.run()
        torch.cuda.synchronize()
        rec = E.tr_profile_read(r.g)
        names = {i: name for name, i in r.vid.items()}
        for x in rec:
            if x["stage"] == "aggregate":                        # only non-contraction vertices still aggregate
                assert r.plan(names[x["vertex"]])["kernel"] not in ("contract_mfma", "contract_alu")
        got = {name: to_host(r.output(name)) for name in r.out_names}
    finally:
        r.close()
    for name in w.outputs:
        bad, worst = violations(got[name].as_f64(), ref[name].as_f64(), rtol_for(w, name))
        assert bad == 0, f"config {n} {pname} output {name}: {bad} elements out of tolerance (worst {worst:.2f}x)"
