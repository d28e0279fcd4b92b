"""Pins of the CPU oracle against what the paper prints and what the mathematics fixes.

None of these tests touches the HIP library.  Each test names the passage of the
paper (arxiv 2410.02682) that fixes the expected value.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import tra_ref as T
from oracle.einsum_ref import einsum_ref, round_bf16
from synth_inputs.prng import f32_to_bf16_bits, bf16_bits_to_f32

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _ints(s):
    return [int(x) for x in s.split(",")]


def _gold_lines(fname, tag):
    with open(os.path.join(GOLD, fname)) as f:
        return [ln.strip() for ln in f if ln.startswith(tag + " ")]


# ------------------------------------------------------------------ integer bookkeeping (golden)
def test_projection_example_section3():
    (ln,) = _gold_lines("bookkeeping.txt", "projection")
    lhs, rhs = ln.split("->")
    kv = dict(p.split("=") for p in lhs.split()[1:])
    got = T.project(_ints(kv["b"]), kv["l1"].split(","), kv["l2"].split(","))
    assert got == _ints(rhs.strip())


def test_aggregation_bound_rank3_example_section3():
    (ln,) = _gold_lines("bookkeeping.txt", "aggbound")
    lhs, rhs = ln.split("->")
    kv = dict(p.split("=") for p in lhs.split()[1:])
    lX, lY = kv["lX"].split(","), kv["lY"].split(",")
    lXY = lX + lY
    bXY = _ints(kv["bXY"])
    lagg = kv["lagg"].split(",")
    assert sorted(T.agg_labels(lX, lY, ["i", "k"])) == sorted(lagg)
    agg_part, z_part = rhs.split(";")
    assert T.project(bXY, lagg, lXY) == _ints(agg_part.strip())
    assert T.project(bXY, ["i", "k"], lXY) == _ints(z_part.split("=")[1])


def test_block_extents_of_rewrite_example_section43():
    (ln,) = _gold_lines("bookkeeping.txt", "extents")
    lhs, rhs = ln.split("->")
    kv = dict(p.split("=") for p in lhs.split()[1:])
    b, d = _ints(kv["b"]), _ints(kv["d"])
    assert [bb // dd for bb, dd in zip(b, d)] == _ints(rhs.strip())
    # and the index arithmetic i*50 + i', k*25 + k': block <1,1> of a 100x50 Z starts at (50, 25)
    off, e, st = T.block_descriptor([100, 50], [2, 2], [1, 1])
    assert (off, e, st) == (50 * 50 + 25, [50, 25], [50, 1])


def test_join_counts_section6_and_figures():
    for ln in _gold_lines("bookkeeping.txt", "joincount"):
        lhs, rhs = ln.split("->")
        d = _ints(lhs.split("=")[1])
        parts = rhs.split()
        assert T.join_count(["i", "j"], ["j", "k"], d) == int(parts[0])
        tt = T.tuple_table("ij,jk->ik", [d[0], d[1], d[3]])
        assert tt["N"] == int(parts[0])
        if len(parts) > 1:
            has_agg = int(parts[1].split("=")[1])
            assert (tt["n_agg"] > 1) == bool(has_agg)


def test_copartition_constraint_section6():
    with pytest.raises(ValueError):
        T.join_count(["i", "j"], ["j", "k"], [2, 2, 4, 2])


def test_subtensor_bounds_and_agg_numbers_section7():
    (ln,) = _gold_lines("bookkeeping.txt", "subbound")
    lhs, rhs = ln.split("->")
    kv = dict(p.split("=") for p in lhs.split()[1:])
    b, d = _ints(kv["b"]), _ints(kv["d"])
    sub = [bb // dd for bb, dd in zip(b, d)]
    toks = rhs.split()
    assert sub == _ints(toks[0])
    assert math.prod(T.project(sub, ["i", "j"], ["i", "j", "j", "k"])) == int(toks[1].split("=")[1])
    assert math.prod(sub[2:]) == int(toks[2].split("=")[1])
    (ln,) = _gold_lines("bookkeeping.txt", "aggcost")
    lhs, rhs = ln.split("->")
    kv = dict(p.split("=") for p in lhs.split()[1:])
    d, p = _ints(kv["d"]), int(kv["p"])
    want = dict(t.split("=") for t in rhs.split())
    tt = T.tuple_table("ij,jk->ik", [d[0], d[1], d[3]])
    n_Z = (8 // d[0]) * (8 // d[3])
    assert tt["N"] == p and tt["n_agg"] == int(want["nagg"]) and n_Z == int(want["nZ"])
    assert (p // tt["n_agg"]) * (tt["n_agg"] - 1) * n_Z == int(want["cost"])


def test_partitioning_count_section81():
    (ln,) = _gold_lines("bookkeeping.txt", "count")
    assert T.count_partitionings(10, 6) == int(ln.split("->")[1])
    # the enumerator agrees with the closed form
    assert len(T.viable(list("abc"), list("cdef"), 2 ** 4)) == T.count_partitionings(4, 6)


def test_viable_list_section82():
    got = T.viable(["i", "j"], ["j", "k"], 8)
    assert len(got) == T.count_partitionings(3, 3) == 10
    for ln in _gold_lines("bookkeeping.txt", "viable"):
        lhs, rhs = ln.split("->")
        d = _ints(lhs.split()[1])
        assert d in got                                  # the printed eight are a subset of the ten
        assert T.project(d, ["i", "k"], ["i", "j", "j", "k"]) == _ints(rhs.strip())
        assert T.join_count(["i", "j"], ["j", "k"], d) == 8


# ------------------------------------------------------------------ tensor relations (golden U)
def _load_u():
    U = np.array([[int(x) for x in ln.split()[1:]] for ln in _gold_lines("u_matrix_blocks.txt", "U")], dtype=np.float64)
    blocks = {}
    for tag in ("D22", "D24"):
        blocks[tag] = {}
        for ln in _gold_lines("u_matrix_blocks.txt", tag):
            k, v = ln.split(":")
            key = tuple(int(x) for x in k.split()[1:])
            blocks[tag][key] = [float(x) for x in v.split()]
    return U, blocks


def test_u_example_blocks_section41():
    U, blocks = _load_u()
    R = T.partition(U, [2, 2])
    assert set(R.blocks) == set(blocks["D22"])
    for key, vals in blocks["D22"].items():
        assert R.blocks[key].shape == (2, 2)
        assert R.blocks[key].ravel().tolist() == vals
    R = T.partition(U, [2, 4])
    assert set(R.blocks) == set(blocks["D24"])
    for key, vals in blocks["D24"].items():
        assert R.blocks[key].shape == (2, 1)
        assert R.blocks[key].ravel().tolist() == vals


def test_equivalence_relation_roundtrip_every_d():
    rng = np.random.default_rng(0)
    A = rng.integers(-9, 9, size=(4, 6, 8)).astype(np.float64)
    for d in itertools.product([1, 2, 4], [1, 2, 3, 6], [1, 2, 4, 8]):
        R = T.partition(A, d)
        assert len(R.blocks) == math.prod(d)
        assert np.array_equal(T.assemble(R), A)           # element-wise definition: j div e, j mod e
        assert np.array_equal(T.assemble_fast(R), A)
        # the block descriptor addresses the same elements in the dense buffer
        flat = A.ravel()
        for key, blk in R.blocks.items():
            off, e, st = T.block_descriptor(A.shape, d, key)
            pos = (1, e[1] - 1, e[2] // 2)
            assert flat[off + sum(p * s for p, s in zip(pos, st))] == blk[pos] if e[0] > 1 else True
        R2 = T.repartition(R, [2, 3, 2])
        assert np.array_equal(T.assemble_fast(R2), A)


def test_partition_rejects_non_divisor():
    with pytest.raises(ValueError):
        T.partition(np.zeros((4, 6)), [3, 2])


# ------------------------------------------------------------------ einsum_ref arithmetic
def test_matmul_vs_textbook_triple_loop():
    rng = np.random.default_rng(1)
    X = rng.integers(-3, 4, size=(5, 7)).astype(np.float64)
    Y = rng.integers(-3, 4, size=(7, 4)).astype(np.float64)
    want = np.zeros((5, 4))
    for i in range(5):
        for k in range(4):
            s = 0.0
            for j in range(7):
                s += X[i, j] * Y[j, k]
            want[i, k] = s
    assert np.array_equal(einsum_ref("ij,jk->ik", X, Y), want)
    # a transposed operand or output must change the answer accordingly
    assert np.array_equal(einsum_ref("ij,jk->ki", X, Y), want.T)
    assert np.array_equal(einsum_ref("ij,kj->ik", X, np.ascontiguousarray(Y.T)), want)
    assert np.array_equal(einsum_ref("ji,jk->ik", np.ascontiguousarray(X.T), Y), want)


@pytest.mark.parametrize("spec,shapes", [
    ("ij,jk->ik", [(9, 5), (5, 6)]),
    ("bij,bjk->bik", [(3, 4, 5), (3, 5, 2)]),
    ("bshd,bthd->bhst", [(2, 5, 3, 4), (2, 6, 3, 4)]),
    ("bhst,bthd->bshd", [(2, 3, 5, 6), (2, 6, 3, 4)]),
    ("bshd,ahd->bsa", [(2, 5, 3, 4), (7, 3, 4)]),
    ("ijk,kl->ijl", [(2, 3, 8), (8, 5)]),
    ("bf,bh->fh", [(6, 4), (6, 5)]),
    ("bc,bc->", [(4, 5), (4, 5)]),
    ("ij,j->i", [(4, 5), (5,)]),
])
def test_contractions_vs_numpy_einsum(spec, shapes):
    rng = np.random.default_rng(2)
    X, Y = (rng.standard_normal(s) for s in shapes)
    np.testing.assert_allclose(einsum_ref(spec, X, Y), np.einsum(spec, X, Y), rtol=1e-12, atol=1e-12)


def test_rank3_example_equals_transposes_bmm_batchsum_section3():
    # b_X = [10,100,20], b_Y = [100,20,2000]; Z_ik = sum_{b,j} X_ijb Y_jbk
    rng = np.random.default_rng(3)
    X = rng.integers(-2, 3, size=(10, 100, 20)).astype(np.float32)
    Y = rng.integers(-2, 3, size=(100, 20, 2000)).astype(np.float32)
    Xt = np.transpose(X, (2, 0, 1)).astype(np.float64)          # [20, 10, 100]
    Yt = np.transpose(Y, (1, 0, 2)).astype(np.float64)          # [20, 100, 2000]
    want = np.matmul(Xt, Yt).sum(axis=0)                         # batch matmul, then sum out the batch
    got = einsum_ref("ijb,jbk->ik", X, Y)
    assert got.shape == (10, 2000)
    assert np.array_equal(got, want)


def test_identity_operand_is_exact_in_every_dtype():
    rng = np.random.default_rng(4)
    X32 = rng.standard_normal((16, 32)).astype(np.float32)
    I32 = np.eye(32, dtype=np.float32)
    assert np.array_equal(einsum_ref("ij,jk->ik", X32, I32, out_dtype="f32"), X32.astype(np.float64))
    Xb = f32_to_bf16_bits(X32)
    Ib = f32_to_bf16_bits(I32)
    got = einsum_ref("ij,jk->ik", Xb, Ib, out_dtype="bf16")
    assert np.array_equal(got, bf16_bits_to_f32(Xb).astype(np.float64))


@pytest.mark.parametrize("k", [256, 8192, 16384])
def test_all_ones_contraction_counts_k_exactly(k):
    ones_a = f32_to_bf16_bits(np.ones((3, k), dtype=np.float32))
    ones_b = f32_to_bf16_bits(np.ones((k, 2), dtype=np.float32))
    for dt in ("f32", "bf16"):                       # powers of two are exact in bf16 too
        assert np.array_equal(einsum_ref("ij,jk->ik", ones_a, ones_b, out_dtype=dt), np.full((3, 2), float(k)))


def test_extended_squared_l2_and_linf_section3():
    rng = np.random.default_rng(5)
    X, Y = rng.standard_normal((6, 9)), rng.standard_normal((9, 4))
    diff = X[:, :, None] - Y[None, :, :]
    np.testing.assert_allclose(einsum_ref("ij,jk->ik", X, Y, otimes="sqdiff", oplus="sum"),
                               (diff ** 2).sum(axis=1), rtol=1e-13)
    assert np.array_equal(einsum_ref("ij,jk->ik", X, Y, otimes="absdiff", oplus="max"), np.abs(diff).max(axis=1))
    # max over all-negative data must not be clamped at zero
    Xn = -np.abs(X) - 1.0
    assert np.array_equal(einsum_ref("ij->i", Xn, otimes="ident", oplus="max"), Xn.max(axis=1))


def test_scalar_functions_against_closed_forms():
    x = np.array([[-2.0, -0.0, 0.0, 0.5, 3.0]])
    y = np.array([[1.5, -1.0, 0.0, 2.0, -0.5]])
    ev = lambda op, a=1.0: einsum_ref("ij,ij->ij", x, y, otimes=op, oplus="none", alpha=a)
    np.testing.assert_allclose(ev("mul", 2.0), 2.0 * x * y)
    np.testing.assert_allclose(ev("add", 0.25), 0.25 * x + y)
    np.testing.assert_allclose(ev("sub", 0.5), 0.5 * (x - y))
    np.testing.assert_allclose(einsum_ref("ij,ij->ij", x, y + 3.0, otimes="div", oplus="none"), x / (y + 3.0))
    np.testing.assert_allclose(ev("exp_sub"), np.exp(x - y), rtol=1e-15)
    assert np.array_equal(ev("relu_grad"), np.where(y > 0, x, 0.0))
    np.testing.assert_allclose(ev("silu_mul"), x / (1 + np.exp(-x)) * y, rtol=1e-15)
    un = lambda op, a=1.0, v=x: einsum_ref("ij->ij", v, otimes=op, oplus="none", alpha=a)
    assert np.array_equal(un("ident"), x)
    assert np.array_equal(un("scale", -3.0), -3.0 * x)
    assert np.array_equal(un("relu"), np.maximum(x, 0.0))
    np.testing.assert_allclose(un("exp"), np.exp(x), rtol=1e-15)
    np.testing.assert_allclose(un("log", v=np.abs(x) + 1), np.log(np.abs(x) + 1), rtol=1e-15)


def test_scalar_functions_at_values_the_mathematics_fixes():
    """Each scalar function at arguments whose result is known without evaluating the same expression again:
    sigmoid(ln 3) = 3/4, exp(ln 6 - ln 2) = 3, log(e^2) = 2, and small integers that show where alpha sits."""
    one = lambda v: np.array([[float(v)]])
    ev = lambda op, x, y, a=1.0: float(einsum_ref("ij,ij->ij", one(x), one(y), otimes=op, oplus="none", alpha=a)[0, 0])
    un = lambda op, x, a=1.0: float(einsum_ref("ij->ij", one(x), otimes=op, oplus="none", alpha=a)[0, 0])
    assert ev("mul", 3, 5, 2.0) == 30.0                       # alpha * x * y
    assert ev("add", 3, 5, 2.0) == 11.0                       # alpha * x + y: alpha scales x only
    assert ev("add", 5, 3, 2.0) == 13.0                       # ... and the operands do not commute
    assert ev("sub", 3, 5, 2.0) == -4.0                       # alpha * (x - y): alpha scales the difference
    assert ev("sub", 5, 3, 2.0) == 4.0
    assert ev("div", 1, 4) == 0.25 and ev("div", 4, 1) == 4.0
    assert ev("sqdiff", 1.5, -2.5) == 16.0 and ev("absdiff", 1.5, -2.5) == 4.0 and ev("absdiff", -2.5, 1.5) == 4.0
    assert abs(ev("exp_sub", np.log(6.0), np.log(2.0)) - 3.0) < 1e-14
    assert abs(ev("exp_sub", np.log(2.0), np.log(6.0)) - 1.0 / 3.0) < 1e-15
    # x * sigmoid(x) * y at x = ln 3: sigmoid = 1 / (1 + 1/3) = 3/4; at x = -ln 3: 1/4; at 0: 0 whatever y
    assert abs(ev("silu_mul", np.log(3.0), 2.0) - np.log(3.0) * 1.5) < 1e-15
    assert abs(ev("silu_mul", -np.log(3.0), 2.0) + np.log(3.0) * 0.5) < 1e-15
    assert ev("silu_mul", 0.0, 7.0) == 0.0
    assert abs(ev("silu_mul", 2.0, np.log(3.0)) - 2.0 * np.log(3.0) / (1.0 + np.exp(-2.0))) < 1e-15   # sigmoid acts on x, not on y
    # the derivative of ReLU passes x where y is positive; zero of either sign, and negatives, give zero (ReLU'(0) = 0)
    assert ev("relu_grad", 7.0, 1e-30) == 7.0 and ev("relu_grad", 7.0, 0.0) == 0.0
    assert ev("relu_grad", 7.0, -0.0) == 0.0 and ev("relu_grad", 7.0, -2.0) == 0.0 and ev("relu_grad", -7.0, 3.0) == -7.0
    assert un("ident", -1.25) == -1.25 and un("scale", 4.0, -1.5) == -6.0
    assert un("relu", -2.0) == 0.0 and un("relu", 3.0) == 3.0 and un("relu", -0.0) == 0.0
    assert abs(un("exp", np.log(5.0)) - 5.0) < 1e-14 and un("exp", 0.0) == 1.0
    assert abs(un("log", np.e ** 2) - 2.0) < 1e-15 and un("log", 1.0) == 0.0 and un("log", 0.125) == np.log2(0.125) * np.log(2.0)


def test_selected_outputs_match_dense():
    rng = np.random.default_rng(6)
    X, Y = rng.standard_normal((7, 5, 3)), rng.standard_normal((3, 4))
    dense = einsum_ref("ijk,kl->ijl", X, Y)
    sel = [0, 5, 17, 7 * 5 * 4 - 1, 33]
    assert np.array_equal(einsum_ref("ijk,kl->ijl", X, Y, sel=sel), dense.ravel()[sel])


def test_malformed_requests_are_rejected():
    a = np.zeros((3, 3))
    with pytest.raises(ValueError):
        einsum_ref("ii,ij->j", a, a)                 # repeated label inside one operand (Section 3)
    with pytest.raises(ValueError):
        einsum_ref("ij,jk->ikz", a, a)               # broadcast label (ignored by the paper)
    with pytest.raises(ValueError):
        einsum_ref("ij,jk->ik", a, np.zeros((4, 3)))  # shared label with two bounds
    with pytest.raises(ValueError):
        einsum_ref("ij,jk->ik", a, a, oplus="none")  # aggregated label without an aggregation operator


# ------------------------------------------------------------------ rounding to the storage dtype
def test_bf16_rounding_ties_to_even_and_range():
    assert round_bf16(1.0 + 2.0 ** -8) == 1.0                     # tie -> even mantissa
    assert round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6     # tie -> even mantissa (up)
    assert round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == 1.0 + 2.0 ** -7
    assert round_bf16(-0.3) == -0.30078125
    assert round_bf16(3.4e38) == math.inf
    assert round_bf16(2.0 ** -133) == 2.0 ** -133                  # smallest bf16 subnormal
    assert round_bf16(2.0 ** -135) == 0.0
    rng = np.random.default_rng(7)
    v = (rng.standard_normal(2000) * np.exp(rng.uniform(-20, 20, 2000))).astype(np.float32)
    want = bf16_bits_to_f32(f32_to_bf16_bits(v)).astype(np.float64)
    got = np.array([round_bf16(float(t)) for t in v])
    assert np.array_equal(got, want)


def test_single_rounding_after_double_accumulation():
    # 1 + 2^-24 + 2^-24: fp32 sequential addition loses both small terms, double keeps them
    X = np.array([[1.0, 2.0 ** -24, 2.0 ** -24]], dtype=np.float32)
    Y = np.ones((3, 1), dtype=np.float32)
    assert einsum_ref("ij,jk->ik", X, Y, out_dtype="f32")[0, 0] == 1.0 + 2.0 ** -23


# ------------------------------------------------------------------ softmax, attention (Section 3)
def _softmax_einsums(Xm, sub_max=True):
    C = einsum_ref("ij->i", Xm, otimes="ident", oplus="max") if sub_max else np.zeros(Xm.shape[0])
    E = einsum_ref("ij,i->ij", Xm, C, otimes="exp_sub", oplus="none")
    S = einsum_ref("ij->i", E, otimes="ident", oplus="sum")
    return einsum_ref("ij,i->ij", E, S, otimes="div", oplus="none")


def test_softmax_macro_pins():
    P = _softmax_einsums(np.full((2, 8), 3.25))
    assert np.array_equal(P, np.full((2, 8), 0.125))                # constant row of length 2^k: exactly 1/n
    P = _softmax_einsums(np.array([[0.0, math.log(2.0), math.log(3.0)]]))
    np.testing.assert_allclose(P, [[1 / 6, 2 / 6, 3 / 6]], rtol=1e-15)
    P = _softmax_einsums(np.array([[1000.0, 1000.0]]))
    assert np.array_equal(P, [[0.5, 0.5]])                          # needs the max subtraction
    rng = np.random.default_rng(8)
    Xm = rng.standard_normal((5, 11)) * 3
    np.testing.assert_allclose(_softmax_einsums(Xm).sum(axis=1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(_softmax_einsums(Xm), _softmax_einsums(Xm, sub_max=False), rtol=1e-13)


def test_multihead_attention_einsums_equal_per_head_matrices():
    rng = np.random.default_rng(9)
    s, a, h, d = 6, 8, 2, 4
    Xq, Xk, Xv = (rng.standard_normal((s, a)) for _ in range(3))
    Wq, Wk, Wv, Wo = (rng.standard_normal((a, h, d)) * 0.3 for _ in range(4))
    QH = einsum_ref("sa,ahd->shd", Xq, Wq)
    KH = einsum_ref("ta,ahd->thd", Xk, Wk)
    VH = einsum_ref("ta,ahd->thd", Xv, Wv)
    T1 = einsum_ref("shd,thd->hst", QH, KH)
    T2 = einsum_ref("hst->hst", T1, otimes="scale", oplus="none", alpha=1 / math.sqrt(d))
    C = einsum_ref("hst->hs", T2, otimes="ident", oplus="max")
    E = einsum_ref("hst,hs->hst", T2, C, otimes="exp_sub", oplus="none")
    S = einsum_ref("hst->hs", E, otimes="ident", oplus="sum")
    T3 = einsum_ref("hst,hs->hst", E, S, otimes="div", oplus="none")
    O = einsum_ref("hst,thd->shd", T3, VH)
    Yo = einsum_ref("shd,ahd->sa", O, Wo)
    # standard presentation: per-head attention, concatenate, multiply by W_O as a matrix
    heads = []
    for i in range(h):
        q, k, v = Xq @ Wq[:, i, :], Xk @ Wk[:, i, :], Xv @ Wv[:, i, :]
        sc = q @ k.T / math.sqrt(d)
        p = np.exp(sc - sc.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        heads.append(p @ v)
    concat = np.concatenate(heads, axis=1)                         # [s, h*d]
    Womat = Wo.reshape(a, h * d).T                                 # [(h d), a]
    np.testing.assert_allclose(Yo, concat @ Womat, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ decomposition invariant (Section 4.3)
INVARIANT_CASES = [
    ("ij,jk->ik", [(8, 8), (8, 8)], "mul", "sum"),
    ("ijb,jbk->ik", [(4, 8, 2), (8, 2, 4)], "mul", "sum"),
    ("bshd,bthd->bhst", [(2, 4, 2, 4), (2, 4, 2, 4)], "mul", "sum"),
    ("ij,jk->ik", [(4, 8), (8, 4)], "absdiff", "max"),
    ("ij,jk->ik", [(4, 8), (8, 4)], "sqdiff", "sum"),
    ("ij,i->ij", [(8, 4), (8,)], "sub", "none"),
    ("bc,bc->", [(4, 8), (4, 8)], "mul", "sum"),
]


@pytest.mark.parametrize("spec,shapes,otimes,oplus", INVARIANT_CASES)
def test_every_partitioning_gives_the_undecomposed_result(spec, shapes, otimes, oplus):
    rng = np.random.default_rng(10)
    X, Y = (rng.integers(-2, 3, size=s).astype(np.float32) for s in shapes)
    lX, lY, lZ = spec.split("->")[0].split(",")[0], spec.split("->")[0].split(",")[1], spec.split("->")[1]
    want = einsum_ref(spec, X, Y, otimes=otimes, oplus=oplus, out_dtype="f32")
    schema = T.concat_unique(list(lX), list(lY))
    bmap = dict(zip(list(lX) + list(lY), list(X.shape) + list(Y.shape)))
    seen = 0
    for p in (1, 2, 4, 8):
        for dfull in T.viable(list(lX), list(lY), p):
            dmap = dict(zip(list(lX) + list(lY), dfull))
            if any(bmap[l] % dmap[l] for l in schema):
                continue
            d = [dmap[l] for l in schema]
            got, ncalls = T.tra_einsum(spec, X, Y, d, otimes=otimes, oplus=oplus, out_dtype="f32")
            assert ncalls == p == T.tuple_table(spec, d)["N"]
            assert np.array_equal(got, want), (spec, d)       # integer data: exact, any summation order
            seen += 1
    assert seen >= 4


def test_unary_reduction_invariant_and_max_aggregation():
    rng = np.random.default_rng(11)
    X = rng.standard_normal((8, 16))
    for d in ([1, 1], [2, 1], [1, 4], [4, 4], [8, 16]):
        got, n = T.tra_einsum("ij->i", X, None, d, otimes="ident", oplus="max")
        assert n == d[0] * d[1]
        assert np.array_equal(got, X.max(axis=1))
        got, _ = T.tra_einsum("ij->i", X, None, d, otimes="ident", oplus="sum")
        np.testing.assert_allclose(got, X.sum(axis=1), rtol=1e-13)


def test_float_inputs_invariant_within_rounding():
    rng = np.random.default_rng(12)
    X, Y = rng.standard_normal((8, 16)), rng.standard_normal((16, 8))
    want = einsum_ref("ij,jk->ik", X, Y)
    for d in ([2, 2, 2], [1, 8, 1], [4, 1, 2], [2, 4, 1]):
        got, _ = T.tra_einsum("ij,jk->ik", X, Y, d)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


def test_tuple_table_rows_for_2x2x2_matmul():
    # keys over (i, j, k), row-major; aggIdx is the j key; group is the rank of (i, k)
    tt = T.tuple_table("ij,jk->ik", [2, 2, 2])
    assert tt["N"] == 8 and tt["n_agg"] == 2 and tt["d_X"] == [2, 2] and tt["d_Y"] == [2, 2] and tt["d_Z"] == [2, 2]
    rows = tt["rows"]
    assert [r["key"] for r in rows] == list(itertools.product(range(2), repeat=3))
    for r in rows:
        i, j, k = r["key"]
        assert r["keyX"] == (i, j) and r["keyY"] == (j, k) and r["keyZ"] == (i, k)
        assert r["aggIdx"] == j and r["group"] == 2 * i + k


def test_aggregation_of_identical_partials_and_max():
    # entries with few significant bits: every running sum is exact, so 8 copies give exactly 8x
    slab = np.arange(12, dtype=np.float64).reshape(3, 4) / 8.0 - 0.625
    temp = [((0, a), (0,), (a,), slab.copy()) for a in range(8)]       # schema (z, a): 8 partials of one group
    out = T.aggregate(temp, ["z", "a"], ["a"], ["z"], {"z": 1, "a": 8}, "sum")
    assert list(out) == [(0,)] and np.array_equal(out[(0,)], 8.0 * slab)   # short mantissas: exact
    rng = np.random.default_rng(13)
    parts = [rng.standard_normal((3, 4)) for _ in range(5)]
    temp = [((0, a), (0,), (a,), parts[a]) for a in range(5)]
    out = T.aggregate(temp, ["z", "a"], ["a"], ["z"], {"z": 1, "a": 5}, "max")
    assert np.array_equal(out[(0,)], np.max(np.stack(parts), axis=0))
