"""Full-size GPU checks, in the launch configuration bench.py times, under EVERY named partitioning of a workload
and under the planner's own labelling (Section 4.3 of the paper: every decomposition computes the undecomposed EinSum).

The oracle cannot evaluate these graphs whole in seconds, so it computes sampled outputs one by one (full reduction
length; rows at tile, block and tail boundaries of all the partitionings) from the same input values.  Its result does
not depend on the partitioning, so what it derives from the inputs alone is computed once per workload and compared
with every partitioning's run.  Where a sampled output needs a whole intermediate tensor that the oracle cannot afford
(the weight gradients of config 3 sum over all 4096 rows of dH1; a row of config 4's output projection needs every
head), the oracle takes that intermediate as the GPU wrote it in the same run, and the intermediate itself is checked
on sampled rows against the oracle's chain from the inputs.  Properties that hold at any size come on top: softmax
rows sum to one, causally masked probabilities are exactly zero.
Config 1 at its full size (256^3) is already compared element by element in test_gpu_parity.py.
"""
import numpy as np
import pytest

from tests._parity import RTOL_BF16, RTOL_F32, violations
from oracle.einsum_ref import einsum_ref
from oracle.graph_ref import to_storage
from synth_inputs import build_config
from synth_inputs.prng import HostTensor

pytestmark = pytest.mark.gpu


def _inputs(n):
    from synth_inputs import prng_torch
    w = build_config(n)
    dev = {v.name: prng_torch.make_tensor(v.recipe, v.bound, v.dtype, w.seed, w.tensor_id(v.name)) for v in w.vertices if v.is_input}
    return w, dev


def _run(w, dev, pname, outputs):
    import torch
    from paper_2410_02682_amd.runner import GraphRunner
    r = GraphRunner(w, pname, outputs=outputs)
    r.bind(dev)
    r.run()
    torch.cuda.synchronize()
    return r


def _setup(n, pname, outputs):
    w, dev = _inputs(n)
    return w, dev, _run(w, dev, pname, outputs)


def _check(what, got, ref, rtol):
    bad, worst = violations(got, ref, rtol)
    assert bad == 0, f"{what}: {bad} out of tolerance (worst {worst:.2f}x)"


def _st(values, dtype):
    """Oracle values (already rounded to dtype) -> the storage array the next oracle call reads."""
    return to_storage(values, dtype).data


def _host(t):
    """Device tensor (or a slice of one) -> numpy array in the oracle's storage convention."""
    import torch
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _f64(arr):
    return HostTensor(arr, "bf16" if arr.dtype == np.uint16 else "f32").as_f64()


def test_config2_matrix_chain_sampled_rows_under_every_partitioning():
    w, dev = _inputs(2)
    # tile and block boundaries of all the partitionings (row blocks of 1024, 2048, 4096 and 8192 rows)
    rows = [0, 255, 256, 1023, 1024, 2047, 2048, 4095, 4096, 8191]
    B, C = _host(dev["B"]), _host(dev["C"])
    ab = einsum_ref("ij,jk->ik", _host(dev["A"][rows]), B, out_dtype="bf16")
    abc = einsum_ref("ik,kl->il", _st(ab, "bf16"), C, out_dtype="f32")
    for pname in list(w.partitionings) + ["eindecomp:8"]:
        print(f"config 2 full size, partitioning {pname}", flush=True)
        r = _run(w, dev, pname, ["AB", "ABC"])
        try:
            assert r.plan("AB")["kernel"] == "contract_mfma"
            if pname == "mix":
                assert r.plan("ABC")["repart_x"] == 1
            _check(f"{pname} AB rows", _f64(_host(r.output("AB")[rows])), ab, RTOL_BF16)
            _check(f"{pname} ABC rows", _f64(_host(r.output("ABC")[rows])), abc, RTOL_BF16)   # downstream of a bf16-rounded intermediate
        finally:
            r.close()


def test_config5_split_reduction_sampled_rows_under_every_partitioning():
    w, dev = _inputs(5)
    Y = _host(dev["Y"])
    picks = [(0, 0), (13, 517), (63, 1023), (31, 255), (32, 256), (31, 1023), (32, 0)]
    refs = [einsum_ref("ijk,kl->ijl", _host(dev["X"][i, j]).reshape(1, 1, -1), Y, out_dtype="f32").ravel() for (i, j) in picks]
    for pname in list(w.partitionings) + ["eindecomp:16"]:
        print(f"config 5 full size, partitioning {pname}", flush=True)
        r = _run(w, dev, pname, None)
        try:
            assert r.plan("Z")["kernel"] == "contract_mfma"
            if pname == "k16":
                assert r.plan("Z")["n_agg"] == 16
            z = r.output("Z")
            for (i, j), ref in zip(picks, refs):
                _check(f"{pname} Z[{i},{j},:]", _f64(_host(z[i, j])), ref, RTOL_F32)
        finally:
            r.close()


def test_config3_ffnn_step_sampled_rows_under_every_partitioning():
    import torch
    w, dev = _inputs(3)
    B = w.dims["b"]
    W1, W2, Yall = _host(dev["W1"]), _host(dev["W2"]), _host(dev["Y"])
    brows = [0, 511, 512, 2047, 2048, 4095]              # batch-block boundaries of the 8-way and the 2-way cut
    # the oracle's chain from the inputs for the sampled batch rows (forward, softmax, and backward down to dA1)
    X_r = _host(dev["X"][brows])
    h1 = einsum_ref("bf,fh->bh", X_r, W1, out_dtype="bf16")
    a1 = einsum_ref("bh->bh", _st(h1, "bf16"), otimes="relu", oplus="none", out_dtype="bf16")
    L = einsum_ref("bh,hc->bc", _st(a1, "bf16"), W2, out_dtype="f32")
    c = einsum_ref("bc->b", _st(L, "f32"), otimes="ident", oplus="max", out_dtype="f32")
    e = einsum_ref("bc,b->bc", _st(L, "f32"), _st(c, "f32"), otimes="exp_sub", oplus="none", out_dtype="f32")
    s = einsum_ref("bc->b", _st(e, "f32"), otimes="ident", oplus="sum", out_dtype="f32")
    p = einsum_ref("bc,b->bc", _st(e, "f32"), _st(s, "f32"), otimes="div", oplus="none", out_dtype="f32")
    dl = einsum_ref("bc,bc->bc", _st(p, "f32"), Yall[brows], otimes="sub", oplus="none", alpha=1.0 / B, out_dtype="bf16")
    da1 = einsum_ref("bc,hc->bh", _st(dl, "bf16"), W2, out_dtype="bf16")
    hrows = [0, 511, 512, 1023, 1024, 4095]              # rows of dW2 (hidden units): block boundaries of h:8 and h:4
    frows = [0, 255, 256, 1023, 1024, 8191]              # rows of dW1 (features)
    for pname in list(w.partitionings) + ["eindecomp:8"]:
        print(f"config 3 full size, partitioning {pname}", flush=True)
        r = _run(w, dev, pname, ["H1", "A1", "L", "P", "loss", "dL", "dH1", "dW1", "dW2"])
        try:
            _check(f"{pname} H1 rows", _f64(_host(r.output("H1")[brows])), h1, RTOL_BF16)
            _check(f"{pname} L rows", _f64(_host(r.output("L")[brows])), L, RTOL_BF16)
            _check(f"{pname} P rows", _f64(_host(r.output("P")[brows])), p, RTOL_BF16)
            _check(f"{pname} dL rows", _f64(_host(r.output("dL")[brows])), dl, RTOL_BF16)
            # ReLU's derivative decides on the sign of the stored H1: both sides take that decision on the same stored
            # values (the GPU's own H1 rows, just compared with the oracle's above)
            dh1 = einsum_ref("bh,bh->bh", _st(da1, "bf16"), _host(r.output("H1")[brows]), otimes="relu_grad", oplus="none", out_dtype="bf16")
            _check(f"{pname} dH1 rows", _f64(_host(r.output("dH1")[brows])), dh1, RTOL_BF16)
            P = r.output("P")
            assert float((P.double().sum(dim=1) - 1.0).abs().max()) < 1e-5          # softmax rows sum to one
            # the loss over all 4096 rows: the oracle's softmax / cross-entropy chain on the logits the GPU wrote
            Lg = _host(r.output("L"))
            cg = einsum_ref("bc->b", Lg, otimes="ident", oplus="max", out_dtype="f32")
            eg = einsum_ref("bc,b->bc", Lg, _st(cg, "f32"), otimes="exp_sub", oplus="none", out_dtype="f32")
            sg = einsum_ref("bc->b", _st(eg, "f32"), otimes="ident", oplus="sum", out_dtype="f32")
            dg = einsum_ref("bc,b->bc", Lg, _st(cg, "f32"), otimes="sub", oplus="none", out_dtype="f32")
            ls = einsum_ref("b->b", _st(sg, "f32"), otimes="log", oplus="none", out_dtype="f32")
            lp = einsum_ref("bc,b->bc", _st(dg, "f32"), _st(ls, "f32"), otimes="sub", oplus="none", out_dtype="f32")
            loss = float(einsum_ref("bc,bc->", Yall, _st(lp, "f32"), alpha=-1.0 / B, out_dtype="f32"))
            got_loss = float(r.output("loss"))
            assert abs(got_loss - loss) <= 1e-5 * abs(loss), (pname, got_loss, loss)
            # the data-parallel gradient sums: sampled rows of dW2 and dW1 over the whole batch, from the activations
            # and gradients the GPU wrote in this run (checked on sampled rows above)
            A1g, dLg = _host(r.output("A1")), _host(r.output("dL"))
            dw2 = einsum_ref("bh,bc->hc", np.ascontiguousarray(A1g[:, hrows]), dLg, out_dtype="f32")
            _check(f"{pname} dW2 rows", _f64(_host(r.output("dW2")[hrows])), dw2, RTOL_BF16)
            Xc = _host(dev["X"][:, frows])
            dw1 = einsum_ref("bf,bh->fh", Xc, _host(r.output("dH1")), out_dtype="f32")
            _check(f"{pname} dW1 rows", _f64(_host(r.output("dW1")[frows])), dw1, RTOL_BF16)
        finally:
            r.close()
        torch.cuda.empty_cache()


_C4_HEADS = [(0, 0), (3, 31), (1, 17)]
_C4_SROWS = [0, 1, 127, 128, 255, 256, 1023, 2047]         # block boundaries of the 8-way cuts of s and of t
_C4_PICKS = [(0, 0), (0, 255), (1, 256), (2, 1023), (3, 1024), (3, 2047)]   # (b, s) rows of the projections and the FFN


def _c4_attention_reference(w, dev):
    """The oracle's chain from the inputs for three (batch entry, head) pairs: Q whole, P and O on sampled query rows."""
    d = w.dims["d"]
    ref = {}
    for (b, h) in _C4_HEADS:
        Xb = _host(dev["X"][b])                            # [s, a]
        Wq, Wk, Wv = (_host(dev[n][:, h, :]) for n in ("Wq", "Wk", "Wv"))
        q = einsum_ref("sa,ad->sd", Xb, Wq, out_dtype="bf16")
        k = einsum_ref("ta,ad->td", Xb, Wk, out_dtype="bf16")
        v = einsum_ref("ta,ad->td", Xb, Wv, out_dtype="bf16")
        t1 = einsum_ref("sd,td->st", _st(q[_C4_SROWS], "bf16"), _st(k, "bf16"), out_dtype="bf16")
        t2 = einsum_ref("st,st->st", _st(t1, "bf16"), _host(dev["M"][_C4_SROWS]), otimes="add", oplus="none", alpha=1.0 / d ** 0.5, out_dtype="bf16")
        t2s = _st(t2, "bf16")
        c = einsum_ref("st->s", t2s, otimes="ident", oplus="max", out_dtype="f32")
        e = einsum_ref("st,s->st", t2s, _st(c, "f32"), otimes="exp_sub", oplus="none", out_dtype="bf16")
        s_ = einsum_ref("st->s", _st(e, "bf16"), otimes="ident", oplus="sum", out_dtype="f32")
        p = einsum_ref("st,s->st", _st(e, "bf16"), _st(s_, "f32"), otimes="div", oplus="none", out_dtype="bf16")
        o = einsum_ref("st,td->sd", _st(p, "bf16"), _st(v, "bf16"), out_dtype="bf16")
        ref[(b, h)] = (q, p, o)
    return ref


def _c4_check_after_attention(pname, r, weights):
    """Output projection and SwiGLU FFN on sampled (b, s) rows: every row crosses all eight 1376-wide blocks of f; the
    oracle starts from the attention output the GPU wrote in this run (checked per head by the caller)."""
    Wo, Wg, Wu, Wd = weights
    bi = [b for b, _ in _C4_PICKS]
    si = [s for _, s in _C4_PICKS]
    Og = _host(r.output("O")[bi, si])                                       # [rows, h, d]
    yatt = einsum_ref("rhd,ahd->ra", Og, Wo, out_dtype="bf16")
    g = einsum_ref("ra,af->rf", _st(yatt, "bf16"), Wg, out_dtype="bf16")
    u = einsum_ref("ra,af->rf", _st(yatt, "bf16"), Wu, out_dtype="bf16")
    hh = einsum_ref("rf,rf->rf", _st(g, "bf16"), _st(u, "bf16"), otimes="silu_mul", oplus="none", out_dtype="bf16")
    out = einsum_ref("rf,fa->ra", _st(hh, "bf16"), Wd, out_dtype="f32")
    for name, want in (("Yatt", yatt), ("G", g), ("U", u), ("Hh", hh), ("Out", out)):
        _check(f"{pname} {name} rows", _f64(_host(r.output(name)[bi, si])), want, RTOL_BF16)


def test_config4_decoder_block_sampled_rows_under_every_partitioning():
    import torch
    w, dev = _inputs(4)
    ref = _c4_attention_reference(w, dev)
    weights = tuple(_host(dev[n]) for n in ("Wo", "Wg", "Wu", "Wd"))
    for pname in list(w.partitionings) + ["eindecomp:8"]:
        print(f"config 4 full size, partitioning {pname}", flush=True)
        r = _run(w, dev, pname, ["Q", "P", "O", "Yatt", "G", "U", "Hh", "Out"])
        try:
            for (b, h) in _C4_HEADS:
                q, p, o = ref[(b, h)]
                _check(f"{pname} Q[{b},:,{h},:]", _f64(_host(r.output("Q")[b, :, h, :])), q, RTOL_BF16)
                _check(f"{pname} P[{b},{h}]", _f64(_host(r.output("P")[b, h][_C4_SROWS])), p, RTOL_BF16)
                _check(f"{pname} O[{b},:,{h},:]", _f64(_host(r.output("O")[b, _C4_SROWS, h, :])), o, RTOL_BF16)
            P = r.output("P")
            assert float((P[0, 0].float().sum(dim=1) - 1.0).abs().max()) < 2e-2     # rows sum to one up to bf16 rounding
            s_len = P.shape[2]
            mask = torch.triu(torch.ones(s_len, s_len, dtype=torch.bool, device=P.device), diagonal=1)
            assert float(P[2, 5][mask].abs().max()) == 0.0                            # future positions: exactly zero
            del mask
            _c4_check_after_attention(pname, r, weights)
        finally:
            r.close()
        torch.cuda.empty_cache()


def test_config4_decoder_block_with_attention_as_one_pass():
    """The same workload with tr_set_fused_attention: the scores, exponentials and probabilities are never stored, so what
    is compared is the attention output (sampled query rows of three heads against the oracle's vertex-by-vertex chain
    from the inputs) and everything after it.  Under `tsplit8` the key label is cut and the group runs on its separate
    vertices, which the launch log must show."""
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner
    w, dev = _inputs(4)
    ref = _c4_attention_reference(w, dev)
    weights = tuple(_host(dev[n]) for n in ("Wo", "Wg", "Wu", "Wd"))
    for pname in w.partitionings:
        print(f"config 4 full size, attention as one pass, partitioning {pname}", flush=True)
        r = GraphRunner(w, pname, outputs=["Q", "O", "Yatt", "G", "U", "Hh", "Out"], fuse_attention=True)
        try:
            r.bind(dev)
            E.tr_profile_enable(r.g, 64)
            r.run()
            torch.cuda.synchronize()
            kernels = [rec["kernel"] for rec in E.tr_profile_read(r.g)]
            assert kernels.count("attention_fused") == (0 if pname == "tsplit8" else 1), (pname, kernels)
            for (b, h) in _C4_HEADS:
                q, _, o = ref[(b, h)]
                _check(f"{pname} Q[{b},:,{h},:]", _f64(_host(r.output("Q")[b, :, h, :])), q, RTOL_BF16)
                _check(f"{pname} O[{b},:,{h},:]", _f64(_host(r.output("O")[b, _C4_SROWS, h, :])), o, RTOL_BF16)
            _c4_check_after_attention(pname, r, weights)
        finally:
            r.close()
        torch.cuda.empty_cache()


def test_config6_skewed_chain_sampled_rows_under_every_partitioning():
    w, dev = _inputs(6)
    # D x E has a reduction over 102400 values: sampled rows at full length, from the inputs, once
    E_ = _host(dev["E"])
    mrows = [0, 511, 512, 1023]
    de = einsum_ref("mn,nk->mk", _host(dev["D"][mrows]), E_, out_dtype="bf16")
    rows = [0, 1279, 1280, 2559, 2560, 5119, 5120, 10239]
    ab = einsum_ref("ij,jk->ik", _host(dev["A"][rows]), _host(dev["B"]), out_dtype="bf16")
    for pname in list(w.partitionings) + ["eindecomp:8"]:
        print(f"config 6 full size, partitioning {pname}", flush=True)
        r = _run(w, dev, pname, ["DE", "Z"])
        try:
            if pname == "splitn8":
                assert r.plan("DE")["n_agg"] == 8 and r.plan("Z")["repart_x"] == 1
            if pname == "eindecomp:8":
                assert r.plan_exact                           # a tree: the dynamic programme's optimum
            _check(f"{pname} DE rows", _f64(_host(r.output("DE")[mrows])), de, RTOL_BF16)
            # the sum, on sampled rows, from the GPU's own DE (checked above on its sampled rows)
            cde = einsum_ref("im,mk->ik", _host(dev["C"][rows]), _host(r.output("DE")), out_dtype="bf16")
            z = einsum_ref("ik,ik->ik", _st(ab, "bf16"), _st(cde, "bf16"), otimes="add", oplus="none", out_dtype="f32")
            _check(f"{pname} Z rows", _f64(_host(r.output("Z")[rows])), z, RTOL_BF16)
        finally:
            r.close()


def test_config7_distances_sampled_rows_under_every_partitioning():
    w, dev = _inputs(7)
    rows = [0, 127, 128, 4095, 4096, 8191]
    X, Y = _host(dev["X"][rows]), _host(dev["Y"])
    Xh, Yh = _host(dev["Xh"][rows]), _host(dev["Yh"])
    table = (("L2", "ij,jk->ik", X, Y, "sqdiff", "sum", "f32"), ("Linf", "ij,jk->ik", X, Y, "absdiff", "max", "f32"),
             ("L2h", "ij,kj->ik", Xh, Yh, "sqdiff", "sum", "f32"), ("Linfh", "ij,kj->ik", Xh, Yh, "absdiff", "max", "bf16"))
    refs = {name: einsum_ref(spec, a, b, otimes=ot, oplus=op, out_dtype=dt) for name, spec, a, b, ot, op, dt in table}
    for pname in w.partitionings:
        print(f"config 7 full size, partitioning {pname}", flush=True)
        r = _run(w, dev, pname, None)
        try:
            for name, spec, a, b, ot, op, dt in table:
                assert r.plan(name)["kernel"] == "contract_alu"
                got = _f64(_host(r.output(name)[rows]))
                if op == "max":
                    # a maximum of exactly representable differences: the fp32 result is exact (bf16: one rounding of it)
                    assert np.array_equal(got, refs[name]), f"{pname} {name}: {int((got != refs[name]).sum())} elements differ"
                else:
                    _check(f"{pname} {name}", got, refs[name], RTOL_F32)
        finally:
            r.close()


def test_blocks_with_more_than_65535_workgroups():
    """One tuple whose block needs more workgroups than one grid dimension holds (the launch then folds the
    position over two grid dimensions): an element-wise vertex, a row reduction and a fused softmax chain, each
    unpartitioned, compared with the oracle on rows at the start, around the fold and at the end."""
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner
    from oracle.graph_ref import run_graph
    from synth_inputs.workloads import Vertex, Workload

    def sm(src, lab):                                      # the softmax chain of Section 3 over the last label
        rows = lab[:-1]
        return [Vertex("Cmax", "f32", spec=f"{lab}->{rows}", otimes="ident", oplus="max", inputs=(src,)),
                Vertex("E", "bf16", spec=f"{lab},{rows}->{lab}", otimes="exp_sub", oplus="none", inputs=(src, "Cmax")),
                Vertex("S", "f32", spec=f"{lab}->{rows}", otimes="ident", oplus="sum", inputs=("E",)),
                Vertex("Z", "bf16", spec=f"{lab},{rows}->{lab}", otimes="div", oplus="none", inputs=("E", "S"))]

    cases = [
        ("map", (17408, 8192), [Vertex("Z", "bf16", spec="ij->ij", otimes="scale", oplus="none", alpha=-1.5, inputs=("X",))],
         "map", 65535 * 256 * 8 // 8192),
        ("row sums", (2228224, 64), [Vertex("Z", "f32", spec="ij->i", otimes="ident", oplus="sum", inputs=("X",))],
         "reduce_row", 65535 * 32),
        ("softmax", (270336, 64), sm("X", "ij"), "softmax_fused", 65535 * 4),
    ]
    for name, shape, vs, kernel, fold in cases:
        print(f"{name} over {shape}, unpartitioned", flush=True)
        w = Workload("large_" + name.replace(" ", "_"), 0, [Vertex("X", "bf16", bound=shape)] + vs, ["Z"], {"whole": {}})
        x = (torch.rand(shape, device="cuda", generator=torch.Generator("cuda").manual_seed(11)) * 2 - 1).to(torch.bfloat16)
        r = GraphRunner(w, "whole")
        try:
            r.bind({"X": x})
            assert r.plan("Z")["n_tuples"] == 1
            E.tr_profile_enable(r.g, 8)
            r.run()
            torch.cuda.synchronize()
            assert [rec["kernel"] for rec in E.tr_profile_read(r.g)] == [kernel]
            assert fold < shape[0]
            rows = sorted(set(list(range(8)) + list(range(fold - 40, min(fold + 40, shape[0]))) + list(range(shape[0] - 8, shape[0]))))
            sub = Workload("rows", 0, [Vertex("X", "bf16", bound=(len(rows),) + shape[1:])] + vs, ["Z"], {"whole": {}})
            ref = run_graph(sub, {"X": HostTensor(_host(x[rows]), "bf16")})["Z"].as_f64()
            got = _f64(_host(r.output("Z")[rows]))
            bad, worst = violations(got, ref, RTOL_BF16 if w.vertex("Z").dtype == "bf16" else RTOL_F32)
            assert bad == 0, f"{name}: {bad} out of tolerance (worst {worst:.2f}x)"
            # every row was written: a pass over all of them that the device can check itself
            z = r.output("Z").float()
            if name == "map":
                assert torch.equal(z, (x.float() * -1.5).to(torch.bfloat16).float())
            elif name == "softmax":
                assert float((z.sum(dim=1) - 1).abs().max()) < 2e-2
            else:
                assert float((z - x.float().sum(dim=1)).abs().max()) < 1e-3
        finally:
            r.close()
        del x, r
        torch.cuda.empty_cache()
