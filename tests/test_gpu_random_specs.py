"""GPU parity on randomly drawn EinSum vertices: label sets, label orders, bounds, partitioning vectors,
scalar functions and dtypes come from a seeded generator, so kernel routes and stride patterns that no
hand-written case names are exercised too.  Every case is compared with the CPU oracle element by element
and, with small-integer inputs under (mul, sum), must be bit-identical to it whatever the partitioning."""
import os

import numpy as np
import pytest

from tests._parity import RTOL_BF16, RTOL_F32, single_vertex, tile_of, violations
from oracle.graph_ref import run_graph
from synth_inputs.prng import HostTensor, small_ints, uniform_pm1

pytestmark = pytest.mark.gpu

N_CASES = int(os.environ.get("EINDECOMP_RANDOM_CASES", "72"))   # more cases on request, same generator
BOUNDS = [1, 2, 3, 4, 6, 8, 12, 16, 24, 40, 64, 72, 136]
BINARY = [("mul", "sum")] * 6 + [("sqdiff", "sum"), ("absdiff", "max"), ("add", "max"), ("sub", "sum"), ("mul", "max")]
UNARY_RED = [("ident", "sum"), ("ident", "max"), ("exp", "sum"), ("relu", "sum"), ("scale", "max")]
UNARY_MAP = ["ident", "scale", "relu", "exp"]
BINARY_MAP = ["mul", "add", "sub", "sqdiff", "absdiff", "exp_sub", "relu_grad", "silu_mul"]


def _divisors(n, cap):
    return [d for d in range(1, min(n, cap) + 1) if n % d == 0]


def draw_case(seed):
    """One random vertex: (spec, bound of X, bound of Y or None, otimes, oplus, alpha, partitioning, in dtype, out dtype)."""
    rng = np.random.default_rng(2410_02682 + seed)
    pool = list("abcdef")
    rng.shuffle(pool)
    kind = ["contract", "contract", "loose", "reduce", "map2", "map1"][seed % 6]
    bound = {}
    if kind == "contract":
        # a matrix product in disguise: labels kept from X alone (rows), from Y alone (columns), shared and summed
        # (contracted), shared and kept (batch); both operands' innermost labels get extents the 16-byte loads of
        # the matrix-core kernels accept, so most of these reach them, with ragged tiles and tails
        roles = ["m"] * int(rng.integers(1, 3)) + ["n"] * int(rng.integers(1, 3)) + ["k"] * int(rng.integers(1, 3)) \
            + ["b"] * int(rng.integers(0, 2))
        role = dict(zip(pool, roles))
        union = pool[:len(roles)]
        lx = [l for l in union if role[l] in "mkb"]
        ly = [l for l in union if role[l] in "nkb"]
        lz = [l for l in union if role[l] in "mnb"]
        rng.shuffle(lx); rng.shuffle(ly); rng.shuffle(lz)
        inner = {lx[-1], ly[-1]}
        budget = 6.0e7
        for l in sorted(union, key=lambda q: q not in inner):
            choices = [b for b in ([8, 16, 24, 40, 64, 72, 136, 264] if l in inner else [1, 2, 3, 4, 6, 12, 40]) if b <= budget]
            bound[l] = int(rng.choice(choices or [1]))
            budget = max(1.0, budget / bound[l])
    elif kind in ("loose", "map2"):
        n_union = int(rng.integers(2, 6))
        union = pool[:n_union]
        if kind == "map2":
            lx = list(union)                                     # an element-wise join: Y's labels are among X's, none aggregated
            ly = [l for l in union if rng.random() < 0.6] or [union[-1]]
            lz = list(union)
        else:
            role = {l: rng.choice(["x", "y", "xy", "xy"]) for l in union}
            lx = [l for l in union if role[l] in ("x", "xy")] or [union[0]]
            ly = [l for l in union if role[l] in ("y", "xy")] or [union[-1]]
            used = [l for l in union if l in lx or l in ly]
            lz = [l for l in used if rng.random() < 0.6]
            if len(lz) == len(used):                              # keep at least one aggregated label
                lz = lz[:-1]
        rng.shuffle(lx); rng.shuffle(ly); rng.shuffle(lz)
    else:
        n_union = int(rng.integers(1, 5))
        lx = pool[:n_union]
        ly = None
        lz = list(lx) if kind == "map1" else [l for l in lx if rng.random() < 0.5]
        if kind == "reduce" and len(lz) == len(lx):
            lz = lz[:-1]
        rng.shuffle(lz)
    labels = list(dict.fromkeys(lx + (ly or [])))
    # bounds: keep the whole index space small enough for the oracle's loop nest
    budget = 2.0e7
    for l in labels:
        if l in bound:
            continue
        choices = [b for b in BOUNDS if b <= budget]
        bound[l] = int(rng.choice(choices))
        budget = max(1.0, budget / bound[l])
    part, p = {}, 1
    for l in labels:
        divs = _divisors(bound[l], 8)
        if kind == "contract" and l in inner:
            divs = [d for d in divs if (bound[l] // d) % 8 == 0]
        d = int(rng.choice(divs))
        if p * d <= 64:
            part[l] = d
            p *= d
    if kind in ("contract", "loose"):
        otimes, oplus = BINARY[int(rng.integers(len(BINARY)))]
    elif kind == "reduce":
        otimes, oplus = UNARY_RED[int(rng.integers(len(UNARY_RED)))]
    elif kind == "map2":
        otimes, oplus = BINARY_MAP[int(rng.integers(len(BINARY_MAP)))], "none"
    else:
        otimes, oplus = UNARY_MAP[int(rng.integers(len(UNARY_MAP)))], "none"
    alpha = float(rng.choice([1.0, 0.5, -2.0])) if otimes in ("scale", "add", "mul") else 1.0
    spec = "".join(lx) + ("," + "".join(ly) if ly is not None else "") + "->" + "".join(lz)
    bx = tuple(bound[l] for l in lx)
    by = tuple(bound[l] for l in ly) if ly is not None else None
    dt_in = "bf16" if rng.random() < 0.6 else "f32"
    dt_out = "bf16" if (dt_in == "bf16" and rng.random() < 0.4) else "f32"
    return spec, bx, by, otimes, oplus, alpha, part, dt_in, dt_out


def _run(w, pname, inputs, contract=None):
    import torch
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    r = GraphRunner(w, pname, contract=contract)
    try:
        r.bind({k: to_device(t) for k, t in inputs.items()})
        r.run()
        torch.cuda.synchronize()
        return to_host(r.output("Z")), r.plan("Z")["kernel"]
    finally:
        r.close()


# 720: a sum of 69696 same-signed terms per output on the one-output-per-lane kernel (needs its compensated summation)
# 259: alpha * x + y under max with the result contiguous along a label of X alone (the operands must not change places)
@pytest.mark.parametrize("seed", sorted(set(range(N_CASES)) | {259, 720}))
def test_random_vertex_matches_oracle(seed):
    spec, bx, by, otimes, oplus, alpha, part, dt_in, dt_out = draw_case(seed)
    print(f"seed {seed}: {spec} X{bx} Y{by} {otimes}/{oplus} alpha {alpha} d {part} {dt_in}->{dt_out}", flush=True)
    x = HostTensor.from_f32(uniform_pm1(500 + seed, 0, int(np.prod(bx))).reshape(bx), dt_in)
    y = None if by is None else HostTensor.from_f32(uniform_pm1(500 + seed, 1, int(np.prod(by))).reshape(by), dt_in)
    w = single_vertex(spec, x, y, dt_out, otimes=otimes, oplus=oplus, alpha=alpha, parts={"d": part, "whole": {}})
    inputs = {"X": x} if y is None else {"X": x, "Y": y}
    ref = run_graph(w, inputs)["Z"]
    rtol = RTOL_BF16 if dt_out == "bf16" else RTOL_F32
    for pname in ("d", "whole"):
        got, kernel = _run(w, pname, inputs)
        assert got.shape == ref.shape
        bad, worst = violations(got.as_f64(), ref.as_f64(), rtol)
        assert bad == 0, f"{pname} ({kernel}): {bad} elements out of tolerance (worst {worst:.2f}x)"


@pytest.mark.parametrize("seed", [s for s in range(N_CASES) if s % 6 in (0, 1, 2)][::2])
def test_random_contraction_on_small_integers_is_bit_identical_to_the_oracle(seed):
    # entries in {-2..2}: every product and partial sum is an integer below 2^24, so fp32 addition is exact in any
    # order and the partitioned result must equal the oracle's bit for bit
    spec, bx, by, _, _, _, part, dt_in, _ = draw_case(seed)
    print(f"seed {seed}: {spec} X{bx} Y{by} integers d {part} {dt_in}", flush=True)
    x = HostTensor.from_f32(small_ints(700 + seed, 0, int(np.prod(bx))).reshape(bx), dt_in)
    y = HostTensor.from_f32(small_ints(700 + seed, 1, int(np.prod(by))).reshape(by), dt_in)
    w = single_vertex(spec, x, y, "f32", parts={"d": part, "whole": {}})
    ref = run_graph(w, {"X": x, "Y": y})["Z"].as_f64()
    for pname in ("d", "whole"):
        got, kernel = _run(w, pname, {"X": x, "Y": y})
        assert np.array_equal(got.as_f64(), ref), f"{pname} ({kernel}) differs from the exact result"


def draw_large_contraction(seed):
    """A contraction large enough for several tiles of the matrix-core kernels in both directions: one or two labels per
    role (rows, columns, contracted, sometimes batch), extents that leave ragged tiles and stage tails, any label
    order in the operands, so both operands can come out contiguous along the contracted label or along rows /
    columns.  About 1e8..3e8 multiply-adds each (a second or so of the oracle)."""
    rng = np.random.default_rng(4_2410_02682 + seed)
    pool = list("abcdefg")
    rng.shuffle(pool)
    roles = ["m"] * int(rng.integers(1, 3)) + ["n"] * int(rng.integers(1, 3)) + ["k"] * int(rng.integers(1, 3)) + ["b"] * int(rng.integers(0, 2))
    role = dict(zip(pool, roles))
    union = pool[:len(roles)]
    lx = [l for l in union if role[l] in "mkb"]
    ly = [l for l in union if role[l] in "nkb"]
    lz = [l for l in union if role[l] in "mnb"]
    rng.shuffle(lx); rng.shuffle(ly); rng.shuffle(lz)
    target = {"m": int(rng.choice([136, 264, 392, 520, 776])), "n": int(rng.choice([136, 264, 392, 520])),
              "k": int(rng.choice([72, 136, 264, 520, 1032])), "b": int(rng.choice([2, 3]))}
    if seed % 4 == 3:                                        # few tiles under thousands of contracted elements
        target.update(m=int(rng.choice([40, 136, 264])), n=int(rng.choice([24, 72, 136])), k=int(rng.choice([4096, 6144, 8192])))
    bound = {}
    for r in "mnkb":
        ls = [l for l in union if role[l] == r]
        if len(ls) == 1:
            bound[ls[0]] = target[r]
        elif len(ls) == 2:                                   # outer x inner = about the target, inner a multiple of 8
            inner = int(rng.choice([8, 24, 40, 64, 96]))
            where = lx if ls[0] in lx else ly                # the label that comes later in its operand is the inner one
            ls.sort(key=where.index)
            bound[ls[0]], bound[ls[1]] = max(2, target[r] // inner), inner
    part, p = {}, 1
    for l in union:
        divs = [d for d in (1, 2, 3, 4) if bound[l] % d == 0 and (bound[l] // d) % 8 == 0]
        d = int(rng.choice(divs or [1]))
        if p * d <= 16:
            part[l] = d
            p *= d
    spec = "".join(lx) + "," + "".join(ly) + "->" + "".join(lz)
    dt_in = "bf16" if rng.random() < 0.7 else "f32"
    dt_out = "bf16" if (dt_in == "bf16" and rng.random() < 0.4) else "f32"
    return spec, tuple(bound[l] for l in lx), tuple(bound[l] for l in ly), part, dt_in, dt_out


@pytest.mark.parametrize("tile", ["", "256x128", "256"])
@pytest.mark.parametrize("seed", range(max(24, N_CASES // 20)))
def test_random_large_contraction_matches_oracle(seed, tile):
    contract = dict(tile=tile_of(tile)) if tile else None    # the larger tiles too, mostly padding at these sizes
    spec, bx, by, part, dt_in, dt_out = draw_large_contraction(seed)
    x = HostTensor.from_f32(uniform_pm1(1300 + seed, 0, int(np.prod(bx))).reshape(bx), dt_in)
    y = HostTensor.from_f32(uniform_pm1(1300 + seed, 1, int(np.prod(by))).reshape(by), dt_in)
    w = single_vertex(spec, x, y, dt_out, parts={"d": part, "whole": {}})
    ref = run_graph(w, {"X": x, "Y": y})["Z"]
    rtol = RTOL_BF16 if dt_out == "bf16" else RTOL_F32
    for pname in ("d", "whole"):
        got, kernel = _run(w, pname, {"X": x, "Y": y}, contract)
        print(f"seed {seed}: {spec} X{bx} Y{by} d {part if pname == 'd' else {}} {dt_in}->{dt_out}: {kernel}", flush=True)
        bad, worst = violations(got.as_f64(), ref.as_f64(), rtol)
        assert bad == 0, f"{pname} ({kernel}): {bad} elements out of tolerance (worst {worst:.2f}x)"
