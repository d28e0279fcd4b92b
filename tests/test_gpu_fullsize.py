"""Full-size GPU checks, in the launch configuration bench.py times.

The oracle cannot evaluate these graphs whole in seconds, so it computes sampled outputs one by one
(full reduction length, tile-boundary and tail rows included) from the same input values, and the
rest is covered by properties that hold at any size: softmax rows sum to one, causally masked
probabilities are exactly zero, and different partitionings of the same graph agree (Section 4.3
of the paper: every decomposition computes the undecomposed EinSum).
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


def _setup(n, pname, outputs):
    import torch
    from paper_2410_02682_amd.runner import GraphRunner
    from synth_inputs import prng_torch
    w = build_config(n)
    dev = {v.name: prng_torch.make_tensor(v.recipe, v.bound, v.dtype, w.seed, w.tensor_id(v.name)) for v in w.vertices if v.is_input}
    r = GraphRunner(w, pname, outputs=outputs)
    r.bind(dev)
    r.run()
    torch.cuda.synchronize()
    return w, dev, r


def _host(t):
    """Device tensor (or a slice of one) -> numpy array in the oracle's storage convention."""
    import torch
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _f64(arr):
    return HostTensor(arr, "bf16" if arr.dtype == np.uint16 else "f32").as_f64()


def test_config2_matrix_chain_sampled_rows():
    print("config 2 full size, partitioning mix", flush=True)
    w, dev, r = _setup(2, "mix", ["AB", "ABC"])
    try:
        assert r.plan("AB")["kernel"] == "contract_mfma" and r.plan("ABC")["repart_x"] == 1
        rows = [0, 255, 256, 4095, 4096, 8191]            # tile and block boundaries of both partitionings
        A = _host(dev["A"][rows])
        B, C = _host(dev["B"]), _host(dev["C"])
        ab = einsum_ref("ij,jk->ik", A, B, out_dtype="bf16")
        got_ab = _f64(_host(r.output("AB")[rows]))
        bad, worst = violations(got_ab, ab, RTOL_BF16)
        assert bad == 0, f"AB rows: {bad} out of tolerance (worst {worst:.2f}x)"
        abc = einsum_ref("ik,kl->il", to_storage(ab, "bf16").data, C, out_dtype="f32")
        got = _f64(_host(r.output("ABC")[rows]))
        bad, worst = violations(got, abc, RTOL_BF16)         # downstream of a bf16-rounded intermediate
        assert bad == 0, f"ABC rows: {bad} out of tolerance (worst {worst:.2f}x)"
    finally:
        r.close()


def test_config5_split_reduction_sampled_rows_and_partition_invariance():
    import torch
    print("config 5 full size, k split 16 ways", flush=True)
    w, dev, r = _setup(5, "k16", None)
    try:
        assert r.plan("Z")["n_agg"] == 16 and r.plan("Z")["kernel"] == "contract_mfma"
        Y = _host(dev["Y"])
        z16 = r.output("Z")
        for (i, j) in [(0, 0), (13, 517), (63, 1023), (31, 255), (32, 256)]:
            x = _host(dev["X"][i, j]).reshape(1, 1, -1)
            ref = einsum_ref("ijk,kl->ijl", x, Y, out_dtype="f32").ravel()
            got = _f64(_host(z16[i, j]))
            bad, worst = violations(got, ref, RTOL_F32)
            assert bad == 0, f"Z[{i},{j},:]: {bad} out of tolerance (worst {worst:.2f}x)"
        z16 = z16.clone()
    finally:
        r.close()
    print("config 5 full size, k unsplit", flush=True)
    from paper_2410_02682_amd.runner import GraphRunner
    r = GraphRunner(w, "k1")
    try:
        r.bind(dev)
        r.run()
        torch.cuda.synchronize()
        z1 = r.output("Z")
        rms = float(z1.double().pow(2).mean().sqrt())
        err = float((z1 - z16).abs().max())
        assert err <= 2 * RTOL_F32 * (rms + float(z1.abs().max())), (err, rms)
    finally:
        r.close()


def test_config3_ffnn_step_sampled_rows_and_properties():
    import torch
    print("config 3 full size, batch split 8 ways", flush=True)
    w, dev, r = _setup(3, "batch8", ["H1", "P", "loss", "dW1", "dW2"])
    try:
        W1, W2 = _host(dev["W1"]), _host(dev["W2"])
        P = r.output("P")
        for b in [0, 511, 512, 4095]:
            x = _host(dev["X"][b:b + 1])
            h1 = einsum_ref("bf,fh->bh", x, W1, out_dtype="bf16")
            bad, worst = violations(_f64(_host(r.output("H1")[b:b + 1])), h1, RTOL_BF16)
            assert bad == 0, f"H1[{b}]: {bad} out of tolerance (worst {worst:.2f}x)"
            a1 = np.maximum(h1, 0.0)
            L = einsum_ref("bh,hc->bc", to_storage(a1, "bf16").data, W2, out_dtype="f32")
            c = einsum_ref("bc->b", L, otimes="ident", oplus="max", out_dtype="f32")
            e = einsum_ref("bc,b->bc", L, c, otimes="exp_sub", oplus="none", out_dtype="f32")
            s = einsum_ref("bc->b", e, otimes="ident", oplus="sum", out_dtype="f32")
            p = einsum_ref("bc,b->bc", e, s, otimes="div", oplus="none", out_dtype="f32")
            bad, worst = violations(_f64(_host(P[b:b + 1])), p, RTOL_BF16)
            assert bad == 0, f"P[{b}]: {bad} out of tolerance (worst {worst:.2f}x)"
        assert float((P.double().sum(dim=1) - 1.0).abs().max()) < 1e-5          # softmax rows sum to one
        # the loss is the mean negative log-probability of the labelled class
        Yl = dev["Y"].float().argmax(dim=1)
        want = float(-(P.double().gather(1, Yl[:, None]).log().mean()))
        assert abs(float(r.output("loss")) - want) < 1e-4 * abs(want)
        dW1, dW2 = r.output("dW1").clone(), r.output("dW2").clone()
    finally:
        r.close()
    print("config 3 full size, hidden split 8 ways", flush=True)
    from paper_2410_02682_amd.runner import GraphRunner
    r = GraphRunner(w, "hidden8", outputs=["dW1", "dW2"])
    try:
        r.bind(dev)
        r.run()
        torch.cuda.synchronize()
        for name, ref in (("dW1", dW1), ("dW2", dW2)):
            got = r.output(name)
            rms = float(ref.double().pow(2).mean().sqrt())
            frac = float(((got - ref).abs() > RTOL_BF16 * (ref.abs() + rms)).float().mean())
            assert frac < 1e-5, f"{name}: partitionings disagree on a fraction {frac} of the elements"
    finally:
        r.close()


def test_config4_decoder_block_sampled_heads_and_properties():
    import torch
    print("config 4 full size, heads split 8 ways", flush=True)
    w, dev, r = _setup(4, "heads8", ["Q", "P", "O", "Out"])
    try:
        d = w.dims["d"]
        for (b, h) in [(0, 0), (3, 31), (1, 17)]:
            Xb = _host(dev["X"][b])                                        # [s, a]
            Wq, Wk, Wv = (_host(dev[n][:, h, :]) for n in ("Wq", "Wk", "Wv"))
            q = einsum_ref("sa,ad->sd", Xb, Wq, out_dtype="bf16")
            k = einsum_ref("ta,ad->td", Xb, Wk, out_dtype="bf16")
            v = einsum_ref("ta,ad->td", Xb, Wv, out_dtype="bf16")
            bad, worst = violations(_f64(_host(r.output("Q")[b, :, h, :])), q, RTOL_BF16)
            assert bad == 0, f"Q[{b},:,{h},:]: {bad} out of tolerance (worst {worst:.2f}x)"
            rows = [0, 1, 127, 128, 1023, 2047]
            qs = to_storage(q[rows], "bf16").data
            t1 = einsum_ref("sd,td->st", qs, to_storage(k, "bf16").data, out_dtype="bf16")
            M = _host(dev["M"][rows])
            t2 = einsum_ref("st,st->st", to_storage(t1, "bf16").data, M, otimes="add", oplus="none", alpha=1.0 / d ** 0.5, out_dtype="bf16")
            t2s = to_storage(t2, "bf16").data
            c = einsum_ref("st->s", t2s, otimes="ident", oplus="max", out_dtype="f32")
            e = einsum_ref("st,s->st", t2s, c.astype(np.float32), otimes="exp_sub", oplus="none", out_dtype="bf16")
            es = to_storage(e, "bf16").data
            s = einsum_ref("st->s", es, otimes="ident", oplus="sum", out_dtype="f32")
            p = einsum_ref("st,s->st", es, s.astype(np.float32), otimes="div", oplus="none", out_dtype="bf16")
            got_p = _f64(_host(r.output("P")[b, h][rows]))
            bad, worst = violations(got_p, p, RTOL_BF16)
            assert bad == 0, f"P[{b},{h}]: {bad} out of tolerance (worst {worst:.2f}x)"
            o = einsum_ref("st,td->sd", to_storage(p, "bf16").data, to_storage(v, "bf16").data, out_dtype="bf16")
            got_o = _f64(_host(r.output("O")[b, rows, h, :]))
            bad, worst = violations(got_o, o, RTOL_BF16)
            assert bad == 0, f"O[{b},:,{h},:]: {bad} out of tolerance (worst {worst:.2f}x)"
        P = r.output("P")
        assert float((P[0, 0].float().sum(dim=1) - 1.0).abs().max()) < 2e-2     # rows sum to one up to bf16 rounding
        s_len = P.shape[2]
        mask = torch.triu(torch.ones(s_len, s_len, dtype=torch.bool, device=P.device), diagonal=1)
        assert float(P[2, 5][mask].abs().max()) == 0.0                            # future positions: exactly zero
        out_heads = r.output("Out").clone()
    finally:
        r.close()
    print("config 4 full size, sequence split 8 ways", flush=True)
    from paper_2410_02682_amd.runner import GraphRunner
    r = GraphRunner(w, "seq8")
    try:
        r.bind(dev)
        r.run()
        torch.cuda.synchronize()
        got = r.output("Out")
        rms = float(out_heads.double().pow(2).mean().sqrt())
        frac = float(((got - out_heads).abs() > RTOL_BF16 * (out_heads.abs() + rms)).float().mean())
        assert frac < 1e-5, f"Out: partitionings disagree on a fraction {frac} of the elements"
    finally:
        r.close()


def test_config6_skewed_chain_sampled_rows_under_two_labellings():
    import torch
    print("config 6 full size, partitioning splitn8", flush=True)
    w, dev, r = _setup(6, "splitn8", ["DE", "Z"])
    try:
        assert r.plan("DE")["n_agg"] == 8 and r.plan("Z")["repart_x"] == 1
        # D x E has a reduction over 102400 values: sampled rows at full length
        E_ = _host(dev["E"])
        mrows = [0, 511, 512, 1023]
        de = einsum_ref("mn,nk->mk", _host(dev["D"][mrows]), E_, out_dtype="bf16")
        bad, worst = violations(_f64(_host(r.output("DE")[mrows])), de, RTOL_BF16)
        assert bad == 0, f"DE rows: {bad} out of tolerance (worst {worst:.2f}x)"
        # the sum, on sampled rows, from the GPU's own DE (already checked above on its sampled rows)
        rows = [0, 1279, 1280, 5119, 5120, 10239]
        ab = einsum_ref("ij,jk->ik", _host(dev["A"][rows]), _host(dev["B"]), out_dtype="bf16")
        cde = einsum_ref("im,mk->ik", _host(dev["C"][rows]), _host(r.output("DE")), out_dtype="bf16")
        z = einsum_ref("ik,ik->ik", to_storage(ab, "bf16").data, to_storage(cde, "bf16").data, otimes="add", oplus="none", out_dtype="f32")
        bad, worst = violations(_f64(_host(r.output("Z")[rows])), z, RTOL_BF16)
        assert bad == 0, f"Z rows: {bad} out of tolerance (worst {worst:.2f}x)"
        z_hand = r.output("Z").clone()
    finally:
        r.close()
    print("config 6 full size, labelled by the planner for p = 8", flush=True)
    from paper_2410_02682_amd.runner import GraphRunner
    r = GraphRunner(w, "eindecomp:8")
    try:
        assert r.plan_exact                               # a tree: the dynamic programme's optimum
        r.bind(dev)
        r.run()
        torch.cuda.synchronize()
        got = r.output("Z")
        rms = float(z_hand.double().pow(2).mean().sqrt())
        frac = float(((got - z_hand).abs() > RTOL_BF16 * (z_hand.abs() + rms)).float().mean())
        assert frac < 1e-5, f"labellings disagree on a fraction {frac} of the elements"
    finally:
        r.close()


def test_config7_distances_sampled_rows():
    print("config 7 full size, partitioning d222", flush=True)
    w, dev, r = _setup(7, "d222", None)
    try:
        for name in ("L2", "Linf", "L2h", "Linfh"):
            assert r.plan(name)["kernel"] == "contract_alu" and r.plan(name)["n_agg"] == 2
        rows = [0, 127, 128, 4095, 4096, 8191]
        X, Y = _host(dev["X"][rows]), _host(dev["Y"])
        Xh, Yh = _host(dev["Xh"][rows]), _host(dev["Yh"])
        for name, spec, a, b, ot, op, dt in (("L2", "ij,jk->ik", X, Y, "sqdiff", "sum", "f32"), ("Linf", "ij,jk->ik", X, Y, "absdiff", "max", "f32"),
                                             ("L2h", "ij,kj->ik", Xh, Yh, "sqdiff", "sum", "f32"), ("Linfh", "ij,kj->ik", Xh, Yh, "absdiff", "max", "bf16")):
            ref = einsum_ref(spec, a, b, otimes=ot, oplus=op, out_dtype=dt)
            got = _f64(_host(r.output(name)[rows]))
            if op == "max":
                # a maximum of exactly representable differences: the fp32 result is exact (bf16: one rounding of it)
                assert np.array_equal(got, ref), f"{name}: {int((got != ref).sum())} elements differ"
            else:
                bad, worst = violations(got, ref, RTOL_F32)
                assert bad == 0, f"{name}: {bad} out of tolerance (worst {worst:.2f}x)"
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
