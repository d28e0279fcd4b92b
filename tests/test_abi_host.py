"""CPU-only tests of the C-ABI library: it loads without a GPU, exports every symbol the header
declares, and its host-side planner reproduces the oracle's tuple tables bit for bit."""
import itertools
import os
import re

import pytest

import paper_2410_02682_amd as E
from paper_2410_02682_amd import _lib
from oracle import tra_ref as T
from synth_inputs import build_config
from synth_inputs.workloads import d_vector

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "eindecomp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int|void|char|size_t|int64_t)\s*\*?\s*([a-z_][a-z0-9_]*)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_loads_and_exports_every_declared_symbol():
    lib = _lib.load()
    declared = _declared_symbols()
    assert {"einsum_graph_create", "tensor_partition", "tr_execute", "tr_aggregate"} <= set(declared)
    for name in declared:
        assert hasattr(lib, name), name
    assert set(_lib.EXPORTS) == set(declared)


def _one_vertex_graph(spec, bx, by, dt="f32", otimes="mul", oplus="sum"):
    g = E.einsum_graph_create()
    ins = [E.einsum_graph_add_input(g, bx, dt)]
    if by is not None:
        ins.append(E.einsum_graph_add_input(g, by, dt))
    v = E.einsum_graph_add_einsum(g, spec, otimes, oplus, 1.0, ins, dt)
    return g, v


PLAN_CASES = [
    ("ij,jk->ik", (8, 8), (8, 8)),
    ("ijb,jbk->ik", (4, 8, 2), (8, 2, 16)),
    ("bshd,bthd->bhst", (2, 4, 2, 8), (2, 8, 2, 8)),
    ("bhst,bthd->bshd", (2, 2, 4, 8), (2, 8, 2, 4)),
    ("bc,bc->", (4, 8), (4, 8)),
    ("ij->i", (8, 16), None),
    ("ij,i->ij", (8, 4), (8,)),
]


@pytest.mark.parametrize("spec,bx,by", PLAN_CASES)
def test_planner_tables_equal_the_literal_join(spec, bx, by):
    lX, lY, lZ = T.split_spec(spec)
    schema = T.concat_unique(lX, lY or [])
    bmap = dict(zip(lX, bx))
    if lY:
        bmap.update(zip(lY, by))
    otimes, oplus = ("mul", "sum") if lY else ("ident", "sum")
    g, v = _one_vertex_graph(spec, bx, by, otimes=otimes, oplus=oplus)
    checked = 0
    for d in itertools.product([1, 2, 4], repeat=len(schema)):
        if any(bmap[l] % dd for l, dd in zip(schema, d)):
            continue
        E.einsum_graph_set_partition(g, v, d)
        got = E.einsum_graph_plan(g, v)
        want = T.tuple_table(spec, d)
        assert got["labels"] == want["schema"]
        assert got["n_tuples"] == want["N"] and got["n_agg"] == want["n_agg"]
        assert got["d_x"] == want["d_X"] and got["d_y"] == want["d_Y"] and got["d_z"] == want["d_Z"]
        assert got["key"] == [r["key"] for r in want["rows"]]
        assert got["key_x"] == [r["keyX"] for r in want["rows"]]
        assert got["key_y"] == [r["keyY"] for r in want["rows"]]
        assert got["key_z"] == [r["keyZ"] for r in want["rows"]]
        assert got["agg_idx"] == [r["aggIdx"] for r in want["rows"]]
        assert got["group"] == [r["group"] for r in want["rows"]]
        # block offsets against the oracle's block descriptors
        bz = [bmap[l] for l in lZ]
        for t, r in enumerate(want["rows"]):
            assert got["off_x"][t] == T.block_descriptor(bx, want["d_X"], r["keyX"])[0]
            if lY:
                assert got["off_y"][t] == T.block_descriptor(by, want["d_Y"], r["keyY"])[0]
            assert got["off_z"][t] == T.block_descriptor(bz, want["d_Z"], r["keyZ"])[0]
        assert got["block_x"] == [b // dd for b, dd in zip(bx, want["d_X"])]
        checked += 1
    assert checked >= 4
    E.einsum_graph_destroy(g)


def test_paper_join_counts_through_the_abi():
    # Section 6: d = [16,2,2,4] gives 128 tuples; Figures 1-2: four vectors with 16 tuples each
    g, v = _one_vertex_graph("ij,jk->ik", (16, 8), (8, 8))
    E.einsum_graph_set_partition(g, v, [16, 2, 4])
    assert E.einsum_graph_plan(g, v)["n_tuples"] == 128
    E.einsum_graph_destroy(g)
    g, v = _one_vertex_graph("ij,jk->ik", (8, 8), (8, 8))
    for d, has_agg in (([4, 1, 4], False), ([2, 1, 8], False), ([2, 4, 2], True), ([2, 2, 4], True)):
        E.einsum_graph_set_partition(g, v, d)
        p = E.einsum_graph_plan(g, v)
        assert p["n_tuples"] == 16 and (p["n_agg"] > 1) == has_agg
    E.einsum_graph_destroy(g)


def test_tensor_relation_blocks_of_the_u_example():
    # Section 4.1: 4x4 U cut d = [2,2]: block <1,0> starts at row 2, column 0 and is 2x2
    rel = E.tensor_partition(0x1000, "f32", [4, 4], [2, 2])
    assert E.tensor_relation_block(rel, [1, 0]) == (8, [2, 2], [4, 1])
    assert E.tensor_relation_block(rel, [0, 1]) == (2, [2, 2], [4, 1])
    E.tensor_relation_destroy(rel)
    rel = E.tensor_partition(0x1000, "f32", [4, 4], [2, 4])
    assert E.tensor_relation_block(rel, [1, 3]) == (11, [2, 1], [4, 1])
    with pytest.raises(E.EgError):
        E.tensor_relation_block(rel, [2, 0])
    E.tensor_relation_destroy(rel)


def test_error_paths_are_detected_on_the_host():
    g = E.einsum_graph_create()
    a = E.einsum_graph_add_input(g, [4, 6], "f32")
    b = E.einsum_graph_add_input(g, [6, 8], "f32")
    c = E.einsum_graph_add_input(g, [5, 8], "f32")
    cases = [
        (dict(spec="ii,jk->ik", ins=[a, b]), -3),        # repeated label
        (dict(spec="ij,jk->ikz", ins=[a, b]), -4),       # broadcast label
        (dict(spec="ij,jk->ik", ins=[a, c]), -5),        # shared label, two bounds
        (dict(spec="ij,jk,kl->il", ins=[a, b]), -2),     # more than two operands
        (dict(spec="ij,jk->ik", ins=[a]), -2),           # operand count
        (dict(spec="ijk,jk->ik", ins=[a, b]), -5),       # rank mismatch
        (dict(spec="ij,jk->ik", ins=[a, 7]), -10),       # unknown input vertex
        (dict(spec="ij,jk->ik", ins=[a, b], oplus="none"), -11),   # aggregated label, no (+)
        (dict(spec="ij,jk->ik", ins=[a, b], otimes="relu"), -11),  # unary function on a binary spec
    ]
    for kw, code in cases:
        with pytest.raises(E.EgError) as ei:
            E.einsum_graph_add_einsum(g, kw["spec"], kw.get("otimes", "mul"), kw.get("oplus", "sum"), 1.0, kw["ins"], "f32")
        assert ei.value.code == code, kw
    v = E.einsum_graph_add_einsum(g, "ij,jk->ik", "mul", "sum", 1.0, [a, b], "f32")
    for d, code in (([2, 2], -6), ([0, 1, 1], -6), ([3, 1, 1], -7), ([1, 4, 1], -7)):
        with pytest.raises(E.EgError) as ei:
            E.einsum_graph_set_partition(g, v, d)
        assert ei.value.code == code
    with pytest.raises(E.EgError):
        E.einsum_graph_set_partition(g, a, [1, 1])       # not an einsum vertex
    with pytest.raises(E.EgError):
        E.tensor_partition(0x1000, "f32", [4, 6], [3, 2])
    with pytest.raises(E.EgError):
        E.tensor_partition(0, "f32", [4, 6], [2, 2])      # NULL device pointer
    # binding errors are caught before any launch
    E.einsum_graph_mark_output(g, v)
    ra = E.tensor_partition(0x1000, "f32", [4, 6], [1, 1])
    rb = E.tensor_partition(0x2000, "f32", [6, 8], [1, 1])
    rc = E.tensor_partition(0x3000, "f32", [5, 8], [1, 1])
    rz_bad = E.tensor_partition(0x4000, "f32", [4, 7], [1, 1])
    with pytest.raises(E.EgError) as ei:
        E.tr_execute(g, [ra, rb], [], 0, 0)
    assert ei.value.code == -10
    with pytest.raises(E.EgError) as ei:
        E.tr_execute(g, [ra, rb, rc], [rz_bad], 0, 0)
    assert ei.value.code == -5
    for r in (ra, rb, rc, rz_bad):
        E.tensor_relation_destroy(r)
    E.einsum_graph_destroy(g)


def test_workspace_accounts_for_partial_slabs_and_reuse():
    g = E.einsum_graph_create()
    a = E.einsum_graph_add_input(g, [64, 64], "bf16")
    b = E.einsum_graph_add_input(g, [64, 64], "bf16")
    ab = E.einsum_graph_add_einsum(g, "ij,jk->ik", "mul", "sum", 1.0, [a, b], "bf16")
    abc = E.einsum_graph_add_einsum(g, "ik,kl->il", "mul", "sum", 1.0, [ab, b], "f32")
    E.einsum_graph_mark_output(g, abc)
    base = E.tr_workspace_bytes(g)
    assert base == 64 * 64 * 2                                    # only the bf16 intermediate
    E.einsum_graph_set_partition(g, ab, [2, 4, 1])                # 4 fp32 partial slabs for AB
    assert E.tr_workspace_bytes(g) == 64 * 64 * 2 + 4 * 64 * 64 * 4
    E.einsum_graph_set_partition(g, abc, [1, 2, 2])               # 2 slabs for ABC reuse AB's slab space
    assert E.tr_workspace_bytes(g) == 64 * 64 * 2 + 4 * 64 * 64 * 4
    p = E.einsum_graph_plan(g, abc)
    assert p["repart_x"] == 1 and p["repart_y"] == 0              # AB produced as [2,1], consumed as [1,2]
    E.einsum_graph_destroy(g)


def test_workspace_spaces_many_large_slabs_apart():
    # more than two partial slabs of at least 1 MiB sit 4 KiB further apart than their dense size
    g = E.einsum_graph_create()
    a = E.einsum_graph_add_input(g, [1024, 512], "bf16")
    b = E.einsum_graph_add_input(g, [512, 1024], "bf16")
    ab = E.einsum_graph_add_einsum(g, "ij,jk->ik", "mul", "sum", 1.0, [a, b], "f32")
    E.einsum_graph_mark_output(g, ab)
    E.einsum_graph_set_partition(g, ab, [1, 2, 1])
    assert E.tr_workspace_bytes(g) == 2 * 1024 * 1024 * 4
    E.einsum_graph_set_partition(g, ab, [1, 8, 1])
    assert E.tr_workspace_bytes(g) == 8 * (1024 * 1024 + 1024) * 4
    E.einsum_graph_destroy(g)


def test_workspace_holds_the_executors_own_pieces():
    """Few outputs under a long reduction: the executor cuts the reduction into pieces of its own, each one more
    partial slab in the workspace (nothing of this shows in the vertex's plan)."""
    def ws(spec, bx, by, d=None, otimes="mul", oplus="sum"):
        g = E.einsum_graph_create()
        ins = [E.einsum_graph_add_input(g, list(bx), "bf16")]
        if by is not None:
            ins.append(E.einsum_graph_add_input(g, list(by), "bf16"))
        z = E.einsum_graph_add_einsum(g, spec, otimes, oplus, 1.0, ins, "f32")
        E.einsum_graph_mark_output(g, z)
        if d:
            E.einsum_graph_set_partition(g, z, d)
        n, plan = E.tr_workspace_bytes(g), E.einsum_graph_plan(g, z)
        E.einsum_graph_destroy(g)
        return n, plan
    # 2 tiles of 128 x 128 under 8192 contracted elements: cut 8 ways (pieces of 1024)
    n, plan = ws("ij,jk->ik", (256, 8192), (8192, 128))
    assert n == 8 * 256 * 128 * 4 and plan["n_agg"] == 1 and plan["n_tuples"] == 1
    # on top of the vertex's own two-way cut: 2 x 4 pieces of 1024
    n, plan = ws("ij,jk->ik", (256, 8192), (8192, 128), [1, 2, 1])
    assert n == 8 * 256 * 128 * 4 and plan["n_agg"] == 2
    # a launch that fills the chip, or a short reduction, is left alone
    assert ws("ij,jk->ik", (4096, 4096), (4096, 4096))[0] == 0
    assert ws("ij,jk->ik", (256, 2048), (2048, 128))[0] == 0
    # one output over 12 M elements: 1024 pieces (the most); 64 columns over 8192 rows: 8 vectors x 8 lane groups x 64 pieces
    assert ws("ij->", (3000, 4096), None, otimes="ident")[0] == 1024 * 4
    assert ws("ij->j", (8192, 64), None, otimes="ident")[0] == 64 * 64 * 4


def test_kernel_routing_of_the_workload_vertices():
    want = {
        2: {"AB": "contract_mfma", "ABC": "contract_mfma"},
        3: {"H1": "contract_mfma", "A1": "map", "L": "contract_mfma", "Cmax": "reduce_row", "E": "map", "S": "reduce_row",
            "loss": "reduce_row", "dW2": "contract_mfma", "dA1": "contract_mfma", "dH1": "map", "dW1": "contract_mfma"},
        4: {"Q": "contract_mfma", "T1": "contract_mfma", "T2": "map", "Cmax": "reduce_row", "O": "contract_mfma",
            "Yatt": "contract_mfma", "Hh": "map", "Out": "contract_mfma"},
        5: {"Z": "contract_mfma"},
        6: {"AB": "contract_mfma", "DE": "contract_mfma", "CDE": "contract_mfma", "Z": "map"},
        7: {"L2": "contract_alu", "Linf": "contract_alu", "L2h": "contract_alu", "Linfh": "contract_alu"},
    }
    for n, kinds in want.items():
        w = build_config(n)
        for pname, part in w.partitionings.items():
            g = E.einsum_graph_create()
            vid = {}
            for v in w.vertices:
                if v.is_input:
                    vid[v.name] = E.einsum_graph_add_input(g, v.bound, v.dtype)
                else:
                    vid[v.name] = E.einsum_graph_add_einsum(g, v.spec, v.otimes, v.oplus, v.alpha, [vid[i] for i in v.inputs], v.dtype)
                    E.einsum_graph_set_partition(g, vid[v.name], d_vector(v.spec, part.get(v.name, {})))
            for name, kind in kinds.items():
                assert E.einsum_graph_plan(g, vid[name])["kernel"] == kind, (n, pname, name)
            E.einsum_graph_destroy(g)


def test_fusion_of_softmax_chains_shrinks_the_workspace_and_can_be_switched_off():
    sizes = {}
    for fuse in (True, False):
        g = E.einsum_graph_create()
        t = E.einsum_graph_add_input(g, [64, 256], "bf16")
        m = E.einsum_graph_add_input(g, [64, 256], "f32")
        t2 = E.einsum_graph_add_einsum(g, "st,st->st", "add", "none", 0.5, [t, m], "bf16")
        c = E.einsum_graph_add_einsum(g, "st->s", "ident", "max", 1.0, [t2], "f32")
        e = E.einsum_graph_add_einsum(g, "st,s->st", "exp_sub", "none", 1.0, [t2, c], "bf16")
        s_ = E.einsum_graph_add_einsum(g, "st->s", "ident", "sum", 1.0, [e], "f32")
        p = E.einsum_graph_add_einsum(g, "st,s->st", "div", "none", 1.0, [e, s_], "bf16")
        E.einsum_graph_mark_output(g, p)
        E.tr_set_fusion(g, fuse)
        sizes[fuse] = E.tr_workspace_bytes(g)
        E.einsum_graph_destroy(g)
    # separately, the scaled scores and their exponentials (and the row statistics) live in the workspace;
    # fused, none of the chain's intermediate tensors exists and the result goes straight to the caller's relation
    assert sizes[True] == 0
    assert sizes[False] >= 2 * 64 * 256 * 2


def _attention_graph(d_head, parts=None, fuse_attention=True, fuse=True, extra_output=None, mask_labels="st", t_len=192):
    """Section 3's attention for 2 x 3 (batch, head) entries as its seven EinSums; returns (graph, vertex ids)."""
    g = E.einsum_graph_create()
    E.tr_set_fusion(g, fuse)
    E.tr_set_fused_attention(g, fuse_attention)
    dims = {"b": 2, "h": 3, "s": 160, "t": t_len, "d": d_head}
    vid = {}
    vid["Q"] = E.einsum_graph_add_input(g, [dims[l] for l in "bshd"], "bf16")
    vid["K"] = E.einsum_graph_add_input(g, [dims[l] for l in "bthd"], "bf16")
    vid["V"] = E.einsum_graph_add_input(g, [dims[l] for l in "bthd"], "bf16")
    vid["M"] = E.einsum_graph_add_input(g, [dims[l] for l in mask_labels], "f32")
    specs = [("T1", "bshd,bthd->bhst", "mul", "sum", 1.0, ("Q", "K"), "bf16"),
             ("T2", f"bhst,{mask_labels}->bhst", "add", "none", d_head ** -0.5, ("T1", "M"), "bf16"),
             ("C", "bhst->bhs", "ident", "max", 1.0, ("T2",), "f32"),
             ("E", "bhst,bhs->bhst", "exp_sub", "none", 1.0, ("T2", "C"), "bf16"),
             ("S", "bhst->bhs", "ident", "sum", 1.0, ("E",), "f32"),
             ("P", "bhst,bhs->bhst", "div", "none", 1.0, ("E", "S"), "bf16"),
             ("O", "bhst,bthd->bshd", "mul", "sum", 1.0, ("P", "V"), "bf16")]
    for name, spec, ot, op, alpha, ins, dt in specs:
        vid[name] = E.einsum_graph_add_einsum(g, spec, ot, op, alpha, [vid[i] for i in ins], dt)
        E.einsum_graph_set_partition(g, vid[name], d_vector(spec, {l: c for l, c in (parts or {}).items() if l in spec}))
    E.einsum_graph_mark_output(g, vid["O"])
    if extra_output:
        E.einsum_graph_mark_output(g, vid[extra_output])
    return g, vid


def test_attention_as_one_pass_keeps_no_intermediate_tensor_where_it_applies():
    """What tr_set_fused_attention decides shows in the workspace size without a GPU: a group it takes needs only the
    classes of the mask's tiles (a byte per 32 queries x 64 keys, four query groups to a word), a group it declines
    needs what the separate vertices need."""
    def size(**kw):
        g, _ = _attention_graph(**kw)
        n = E.tr_workspace_bytes(g)
        E.einsum_graph_destroy(g)
        return n
    scores = 2 * 3 * 160 * 192 * 2                      # one bf16 tensor of the scores' shape
    table = 256                                         # 8 query groups x 3 key blocks = 24 bytes, rounded to the arena's granule
    for d_head in (32, 64, 128):
        assert size(d_head=d_head) == table
        assert size(d_head=d_head, parts={"b": 2, "h": 3, "s": 5}) == table      # cuts of batch and query labels are views
    unfused = size(d_head=64, fuse_attention=False)
    assert unfused >= scores                            # the scores at least (the softmax chain itself still runs as one pass)
    # declined: the key label or the head dimension is cut, the head dimension has no variant, an intermediate is wanted,
    # softmax fusion is off altogether, the added operand carries a batch label
    assert size(d_head=64, parts={"t": 2}) >= scores
    assert size(d_head=64, parts={"d": 2}) >= scores
    assert size(d_head=48) == size(d_head=48, fuse_attention=False) >= scores
    assert size(d_head=64, extra_output="P") >= scores
    assert size(d_head=64, extra_output="C") >= scores
    assert size(d_head=64, fuse=False) >= 3 * scores
    assert size(d_head=64, mask_labels="hst") >= scores
    with pytest.raises(E.EgError):
        E.tr_set_fused_attention(None, True)



def _xent_graph(fuse=True, outputs=("loss", "dL"), row_cut=1, class_cut=1, late_y=False):
    """Softmax over c followed by log-probabilities, loss and gradient (config 3's vertices around the loss) on 64 x 512."""
    g = E.einsum_graph_create()
    E.tr_set_fusion(g, fuse)
    vid = {"L": E.einsum_graph_add_input(g, [64, 512], "f32"), "Y0": E.einsum_graph_add_input(g, [64, 512], "bf16")}
    specs = [("C", "bc->b", "ident", "max", 1.0, ("L",), "f32"),
             ("E", "bc,b->bc", "exp_sub", "none", 1.0, ("L", "C"), "f32"),
             ("S", "bc->b", "ident", "sum", 1.0, ("E",), "f32"),
             ("P", "bc,b->bc", "div", "none", 1.0, ("E", "S"), "f32"),
             ("D", "bc,b->bc", "sub", "none", 1.0, ("L", "C"), "f32"),
             ("logS", "b->b", "log", "none", 1.0, ("S",), "f32"),
             ("logP", "bc,b->bc", "sub", "none", 1.0, ("D", "logS"), "f32"),
             ("Y", "bc->bc", "scale", "none", 1.0, ("Y0",), "bf16"),
             ("loss", "bc,bc->", "mul", "sum", -1.0 / 64, ("Y", "logP"), "f32"),
             ("dL", "bc,bc->bc", "sub", "none", 1.0 / 64, ("P", "Y"), "bf16")]
    if not late_y:                                  # the labels as a vertex in front of the chain: a tensor the pass can read
        specs.insert(0, specs.pop(7))
    for name, spec, ot, op, alpha, ins, dt in specs:
        vid[name] = E.einsum_graph_add_einsum(g, spec, ot, op, alpha, [vid[i] for i in ins], dt)
        cut = {"b": row_cut, "c": class_cut if name in ("C", "E", "S", "P") else 1}
        E.einsum_graph_set_partition(g, vid[name], d_vector(spec, {l: c for l, c in cut.items() if l in spec and c > 1}))
    for o in outputs:
        E.einsum_graph_mark_output(g, vid[o])
    return g, vid


def test_tails_of_a_softmax_chain_are_laid_out_only_where_somebody_reads_them():
    """Which element-wise vertices the softmax pass evaluates itself shows in the workspace size without a GPU: D, log S and
    the probabilities exist nowhere when only tails read them; the log-probabilities are kept for the loss; a vertex whose
    operand is produced after the chain, or a chain whose softmax label is cut, runs as before."""
    def size(**kw):
        g, _ = _xent_graph(**kw)
        n = E.tr_workspace_bytes(g)
        E.einsum_graph_destroy(g)
        return n
    full, labels = 64 * 512 * 4, 64 * 512 * 2
    def about(n, expected):                                                   # (+ the few partial sums the loss is cut into)
        return expected <= n < expected + 8192
    assert about(size(), labels + full)                                       # Y (a vertex of its own) and logP, nothing else
    assert about(size(row_cut=8), labels + full)                              # cuts of the row label are views
    assert about(size(outputs=("loss", "dL", "logP")), labels)                # an output lives in the caller's relation
    assert about(size(outputs=("loss", "dL", "P", "D")), labels + full)       # asked for: written to the caller's relations
    separate = size(fuse=False)
    assert separate >= labels + 3 * full                                      # E, P (or D) and logP at the least
    # the labels produced after the division: dL cannot join the pass, so the probabilities are stored for it
    assert size(late_y=True) >= labels + 2 * full
    # the softmax label cut: no chain, no tails
    assert size(class_cut=2) == size(class_cut=2, fuse=False)
