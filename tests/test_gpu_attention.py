"""Parity of the one-pass attention (tr_set_fused_attention) with the oracle's evaluation of the same graph vertex by
vertex: Section 3's attention written as a contraction over the head dimension, alpha * x + mask, the four softmax
EinSums over the key label, and the contraction with V.  Ragged query and key counts (several 128-query blocks and
64-key blocks with tails), all three head dimensions, operand layouts with the labels in different orders, with and
without a mask, fp32 and bf16 scores and results, partitioned batch / query labels; the cases the pass must decline
(key label or head dimension cut, a second consumer of an intermediate) must still come out right on the separate
vertices."""
import numpy as np
import pytest

from tests._parity import RTOL_BF16, violations
from oracle.graph_ref import run_graph
from synth_inputs.prng import HostTensor, causal_mask, normal, uniform_pm1
from synth_inputs.workloads import Vertex, Workload

pytestmark = pytest.mark.gpu


def attention_graph(q_spec, k_spec, v_spec, o_spec, dims, mask=None, t_dtype="bf16", o_dtype="bf16", parts=None, extra_output=None,
                    mask_dtype="f32"):
    """q_spec etc.: label strings of Q, K, V and the result over b, h (batch), s, t, d; the scores are (batch..)st.
    mask: None or the label string of the added operand."""
    batch = "".join(l for l in "bh" if l in q_spec)
    z = batch + "st"
    shape = lambda labels: tuple(dims[l] for l in labels)
    vs = [Vertex("Q", "bf16", bound=shape(q_spec)), Vertex("K", "bf16", bound=shape(k_spec)), Vertex("V", "bf16", bound=shape(v_spec))]
    alpha = 1.0 / dims["d"] ** 0.5
    if mask:
        vs.append(Vertex("M", mask_dtype, bound=shape(mask)))
        vs.append(Vertex("T1", t_dtype, spec=f"{q_spec},{k_spec}->{z}", inputs=("Q", "K")))
        vs.append(Vertex("T2", t_dtype, spec=f"{z},{mask}->{z}", otimes="add", oplus="none", alpha=alpha, inputs=("T1", "M")))
        src = "T2"
    else:
        vs.append(Vertex("T1", t_dtype, spec=f"{q_spec},{k_spec}->{z}", alpha=alpha, inputs=("Q", "K")))
        src = "T1"
    vs += [
        Vertex("Cmax", "f32", spec=f"{z}->{z[:-1]}", otimes="ident", oplus="max", inputs=(src,)),
        Vertex("E", "bf16", spec=f"{z},{z[:-1]}->{z}", otimes="exp_sub", oplus="none", inputs=(src, "Cmax")),
        Vertex("S", "f32", spec=f"{z}->{z[:-1]}", otimes="ident", oplus="sum", inputs=("E",)),
        Vertex("P", "bf16", spec=f"{z},{z[:-1]}->{z}", otimes="div", oplus="none", inputs=("E", "S")),
        Vertex("O", o_dtype, spec=f"{z},{v_spec}->{o_spec}", inputs=("P", "V")),
    ]
    outputs = ["O"] + ([extra_output] if extra_output else [])
    p = {"d": {v.name: {l: c for l, c in (parts or {}).items() if l in v.spec} for v in vs if not v.is_input}}
    return Workload("attention", 77, vs, outputs, p, dict(dims))


def inputs_of(w, mask_kind):
    ins = {}
    for i, v in enumerate(w.vertices):
        if not v.is_input:
            continue
        n = int(np.prod(v.bound))
        if v.name == "M":
            if mask_kind == "causal":
                m = causal_mask(*v.bound)
            else:                                       # finite biases with a tenth of the entries at -inf, never a whole row
                m = uniform_pm1(w.seed, i, n).reshape(v.bound).copy()
                hole = uniform_pm1(w.seed, 100 + i, n).reshape(v.bound) > 0.8
                hole[..., 0] = False
                m[hole] = -np.inf
                if mask_kind == "dead_row" and len(v.bound) == 2:
                    m[min(5, v.bound[0] - 1), :] = -np.inf     # one query with no admissible key: NaN on both sides
            ins[v.name] = HostTensor.from_f32(m, v.dtype)
        else:
            ins[v.name] = HostTensor.from_f32(normal(w.seed, i, n, 1.0).reshape(v.bound), "bf16")
    return ins


def run_fused(w, ins, outputs=("O",), fuse_attention=True):
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    r = GraphRunner(w, "d", outputs=list(outputs), fuse_attention=fuse_attention)
    try:
        r.bind({k: to_device(t) for k, t in ins.items()})
        E.tr_profile_enable(r.g, 64)
        r.run()
        torch.cuda.synchronize()
        kernels = [rec["kernel"] for rec in E.tr_profile_read(r.g)]
        got = {n: to_host(r.output(n)) for n in outputs}
    finally:
        r.close()
    return got, kernels


def check(got, ref, name="O"):
    g, r = got[name].as_f64(), ref[name].as_f64()
    assert np.array_equal(np.isnan(g), np.isnan(r)), "NaN entries differ"
    rep = {}
    bad, worst = violations(np.nan_to_num(g, nan=0.0), np.nan_to_num(r, nan=0.0), RTOL_BF16, report=rep)
    assert bad == 0, f"{bad} elements out of tolerance (worst {worst:.2f}x)"
    assert rep["strict_worst"] <= RTOL_BF16, rep


# q, k, v, o label orders; dims; mask labels; mask kind; scores dtype; result dtype; partitioning
CASES = [
    # the decoder block's layout: heads between the token label and the head dimension
    ("bshd", "bthd", "bthd", "bshd", dict(b=2, h=3, s=300, t=300, d=128), "st", "causal", "bf16", "bf16", None),
    ("bshd", "bthd", "bthd", "bshd", dict(b=2, h=4, s=300, t=300, d=128), "st", "causal", "bf16", "bf16", {"h": 2, "s": 2}),
    # keys and queries of different counts, no mask, head-major layout
    ("bhsd", "bhtd", "bhtd", "bhsd", dict(b=1, h=5, s=200, t=330, d=64), None, None, "bf16", "f32", None),
    ("bhsd", "bhtd", "bhtd", "bshd", dict(b=2, h=2, s=129, t=65, d=32), "st", "random", "f32", "bf16", {"b": 2}),
    # one batch label; the mask stored key-major (strided along the key label), and a mask over the keys only
    ("hsd", "htd", "htd", "shd", dict(h=3, s=77, t=500, d=128), "ts", "random", "bf16", "bf16", None),
    ("hsd", "htd", "htd", "hsd", dict(h=2, s=260, t=100, d=64), "t", "random", "bf16", "f32", None),
    # no batch label at all; a query row that is masked out entirely
    ("sd", "td", "td", "sd", dict(s=140, t=70, d=32), "st", "dead_row", "f32", "f32", None),
    ("sd", "td", "td", "sd", dict(s=1, t=1, d=128), None, None, "bf16", "bf16", None),
    ("sd", "td", "td", "sd", dict(s=128, t=64, d=64), "st", "causal", "bf16", "bf16", None),
]


@pytest.mark.parametrize("q,k,v,o,dims,mask,mask_kind,t_dtype,o_dtype,parts", CASES)
def test_attention_in_one_pass_matches_the_oracle(q, k, v, o, dims, mask, mask_kind, t_dtype, o_dtype, parts):
    print(f"one-pass attention {q},{k},{v}->{o} {dims} mask {mask}/{mask_kind} scores {t_dtype} result {o_dtype} d {parts}", flush=True)
    w = attention_graph(q, k, v, o, dims, mask, t_dtype, o_dtype, parts)
    ins = inputs_of(w, mask_kind)
    ref = run_graph(w, ins)
    got, kernels = run_fused(w, ins)
    assert kernels == ["attention_fused"], kernels
    check(got, ref)
    # and the separate vertices on the same inputs, for the record of how far the two device paths are apart
    sep, kernels = run_fused(w, ins, fuse_attention=False)
    assert "attention_fused" not in kernels
    check(sep, ref)


DECLINED = [
    # the key label cut: row maxima and sums are aggregated over partial blocks; the pass must leave the group alone
    (dict(parts={"t": 2}), ("O",)),
    # the head dimension cut at the contractions
    (dict(parts={"d": 2}), ("O",)),
    # the probabilities are an output of the graph as well
    (dict(extra_output="P"), ("O", "P")),
    (dict(extra_output="Cmax"), ("O", "Cmax")),
]


@pytest.mark.parametrize("kw,outputs", DECLINED)
def test_groups_the_pass_cannot_take_run_on_the_separate_vertices(kw, outputs):
    print(f"attention group that must be declined: {kw}", flush=True)
    w = attention_graph("bshd", "bthd", "bthd", "bshd", dict(b=1, h=2, s=150, t=150, d=64), "st", "bf16", "bf16", **kw)
    ins = inputs_of(w, "causal")
    ref = run_graph(w, ins)
    got, kernels = run_fused(w, ins, outputs=outputs)
    assert "attention_fused" not in kernels, kernels
    for n in outputs:
        check(got, ref, n)


def test_mask_stored_as_bf16():
    print("one-pass attention with a bf16 mask", flush=True)
    w = attention_graph("bhsd", "bhtd", "bhtd", "bhsd", dict(b=2, h=2, s=190, t=256, d=64), "st", mask_dtype="bf16")
    ins = inputs_of(w, "random")
    ref = run_graph(w, ins)
    got, kernels = run_fused(w, ins)
    assert kernels == ["attention_fused"], kernels
    check(got, ref)


def test_operands_the_pass_cannot_address_are_refused_before_anything_runs():
    """A group the structural test takes, bound to a V whose head dimension is not contiguous: tr_execute reports
    EG_ERR_LIMIT (the message says which switch to turn off) and has launched nothing."""
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    print("one-pass attention bound to a V with a strided head dimension", flush=True)
    w = attention_graph("hsd", "htd", "htd", "hsd", dict(h=2, s=64, t=64, d=64))
    ins = inputs_of(w, None)
    dev = {k: to_device(t) for k, t in ins.items()}
    dev["V"] = dev["V"].transpose(1, 2).contiguous().transpose(1, 2)           # same values, d no longer the fastest label
    for fuse_attention, fails in ((True, True), (False, False)):
        r = GraphRunner(w, "d", fuse_attention=fuse_attention)
        try:
            r.bind(dev)
            out = r.output("O")
            out.fill_(7.0)
            torch.cuda.synchronize()
            if fails:
                with pytest.raises(E.EgError) as err:
                    r.run()
                assert err.value.code == -13 and "tr_set_fused_attention" in str(err.value)      # EG_ERR_LIMIT
                torch.cuda.synchronize()
                assert bool((out == 7.0).all())
            else:
                r.run()
                torch.cuda.synchronize()
                check({"O": to_host(out)}, run_graph(w, ins))
        finally:
            r.close()


def test_decoder_block_with_one_pass_attention():
    """The small decoder block (Section 3's attention between its projections, then the gated feed-forward block) under
    every partitioning.  Where the key label is not cut the attention runs as one launch and its result O matches the
    oracle's within the bf16 bound.  The separate vertices round exactly where the oracle rounds, so their O is the
    oracle's almost bit for bit; the pass's O carries an error of its own (smaller against exact attention, but
    independent of the oracle's), which four further bf16-rounded stages would be compared with at every element
    above the rms if the block's output were held against the oracle's directly.  The rest of the block is therefore
    checked against the oracle evaluated FROM the device's O: it must match as closely as any other graph."""
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    from synth_inputs import build_config, make_tensor
    w = build_config(4, small=True)
    ins = {v.name: make_tensor(v.recipe, v.bound, v.dtype, w.seed, w.tensor_id(v.name)) for v in w.vertices if v.is_input}
    ref = run_graph(w, ins)
    tail_names = ["Yatt", "G", "U", "Hh", "Out"]
    tail_inputs = ["Wo", "Wg", "Wu", "Wd"]
    tail = Workload("decoder_block_after_attention", w.seed,
                    [w.vertex(n) for n in tail_inputs] + [Vertex("O", "bf16", bound=ref["O"].shape)] + [w.vertex(n) for n in tail_names], ["Out"])
    for pname in w.partitionings:
        print(f"decoder block, partitioning {pname}", flush=True)
        r = GraphRunner(w, pname, outputs=["O", "Out"], fuse_attention=True)
        try:
            r.bind({k: to_device(t) for k, t in ins.items()})
            E.tr_profile_enable(r.g, 64)
            r.run()
            torch.cuda.synchronize()
            kernels = [rec["kernel"] for rec in E.tr_profile_read(r.g)]
            got = {n: to_host(r.output(n)) for n in ("O", "Out")}
        finally:
            r.close()
        assert ("attention_fused" in kernels) == (pname != "tsplit8"), (pname, kernels)
        check(got, ref, "O")
        ref_tail = run_graph(tail, dict({n: ins[n] for n in tail_inputs}, O=got["O"]))
        check(got, ref_tail, "Out")
