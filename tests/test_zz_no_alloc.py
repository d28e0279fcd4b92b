"""tr_execute_static (the entry point for callers that cannot allocate: it keeps partial slabs and intermediates in a
static device array of the library) against tr_execute, through the C ABI: same kernels in the same order, so the
results must be the same bits.  Two calls in a row, the second on a smaller graph, so that what the first call left in
the shared array is there when the second runs.  Runs last in the suite and also alone in a fresh process."""
import numpy as np
import pytest

from oracle.graph_ref import make_inputs, run_graph
from synth_inputs import build_config
from tests._parity import rtol_for, violations

pytestmark = pytest.mark.gpu


def _both(w, pname, inp):
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device, to_host
    dev = {k: to_device(t) for k, t in inp.items()}
    out = {}
    for static in (False, True):
        r = GraphRunner(w, pname)
        try:
            r.bind(dev, workspace=not static)
            need = r.workspace_bytes
            assert 0 < need <= E.tr_static_workspace_bytes(), need
            before = torch.cuda.memory_allocated()
            if static:
                r.run_static()
                assert torch.cuda.memory_allocated() == before
            else:
                r.run()
            torch.cuda.synchronize()
            out[static] = {n: to_host(r.output(n)) for n in r.out_names}
        finally:
            r.close()
    return out[False], out[True], need


def test_static_workspace_entry_point_matches_tr_execute_on_two_calls_in_a_row():
    import paper_2410_02682_amd as E
    assert E.tr_static_workspace_bytes() == 32 << 20
    sizes = []
    # first the small FFNN step (16 einsum vertices: intermediates, partial slabs of the gradient sums, a fused softmax
    # pass, split reductions), then the smaller matrix chain, then config 1 at its full size: each call finds the
    # previous one's bytes in the array
    for n, pname in ((3, "batch8"), (2, "mix"), (1, "d222")):
        print(f"config {n} small, partitioning {pname}: tr_execute, then tr_execute_static", flush=True)
        w = build_config(n, small=True)
        inp = make_inputs(w)
        plain, static, need = _both(w, pname, inp)
        sizes.append(need)
        ref = run_graph(w, inp)
        for name in w.outputs:
            assert np.array_equal(static[name].data, plain[name].data), f"config {n} output {name}: tr_execute_static differs from tr_execute"
            bad, worst = violations(static[name].as_f64(), ref[name].as_f64(), rtol_for(w, name))
            assert bad == 0, f"config {n} output {name}: {bad} elements out of tolerance against the oracle (worst {worst:.2f}x)"
    assert sizes[0] > sizes[1] > sizes[2], sizes


def test_static_workspace_entry_point_rejects_graphs_beyond_its_limit():
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner
    w = build_config(2, dims={"i": 4096, "j": 4096, "k": 4096, "l": 4096})       # AB alone is 32 MiB, the partial slabs 128 MiB
    r = GraphRunner(w, "mix")
    try:
        dev = {v.name: torch.zeros(v.bound, dtype=torch.bfloat16, device="cuda") for v in w.vertices if v.is_input}
        r.bind(dev, workspace=False)
        assert r.workspace_bytes > E.tr_static_workspace_bytes()
        out = r.output("ABC")
        out.fill_(7.0)
        torch.cuda.synchronize()
        with pytest.raises(E.EgError) as e:
            r.run_static()
        assert e.value.code == -9 and "static workspace" in str(e.value)
        torch.cuda.synchronize()
        assert float(out.min()) == 7.0 and float(out.max()) == 7.0                  # nothing was launched
    finally:
        r.close()
