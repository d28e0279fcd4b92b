#!/usr/bin/env python3
"""Benchmark of the tensor-relational einsum hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: tr_execute of the
matrix-chain graph (A.B).C with i=j=k=l=8192, bf16 storage, fp32 accumulation, the first product
cut (2,2,2) and the second (1,2,4): two joins of 8 block contractions each on MFMA, each followed
by the aggregation of two fp32 partial slabs, with a repartition of A.B in between.  Inputs are
resident in HBM before the timed region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def cpu_baseline(w, inp, budget_s=15.0):
    """Times the oracle as it stands on a bounded sample: R rows of the first product at full reduction length."""
    import numpy as np
    from oracle.einsum_ref import einsum_ref
    A, B = inp["A"].data, inp["B"].data
    j, k = B.shape

    def run(rows):
        t0 = time.perf_counter()
        einsum_ref("ij,jk->ik", A[:rows], B, out_dtype="bf16", x_dtype="bf16", y_dtype="bf16")
        return time.perf_counter() - t0

    t = run(8)                                        # calibration
    rows = int(max(8, min(A.shape[0], 8 * budget_s / max(t, 1e-3))))
    t = run(rows)
    flops = 2.0 * rows * j * k
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": flops / t / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{rows} of {A.shape[0]} rows of A.B at full reduction length {j} (einsum_ref, double accumulation), {t:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--partitioning", default="mix")
    ap.add_argument("--size", type=int, default=8192, help="side of every matrix in the chain")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner, to_device
    from synth_inputs import build_config
    from synth_inputs.prng import make_tensor

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    n = args.size
    w = build_config(2, dims={"i": n, "j": n, "k": n, "l": n})
    inp = {v.name: make_tensor(v.recipe, v.bound, v.dtype, w.seed, w.tensor_id(v.name)) for v in w.vertices if v.is_input}
    r = GraphRunner(w, args.partitioning)
    r.bind({k: to_device(t) for k, t in inp.items()})
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        r.run(stream)
    torch.cuda.synchronize()
    launches_per_step = sum(2 if r.plan(v.name)["n_agg"] > 1 else 1 for v in w.einsum_vertices())
    E.tr_profile_enable(r.g, launches_per_step * args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        r.run(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    rec = E.tr_profile_read(r.g)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops_per_step = 2.0 * 2.0 * n * n * n
    value = flops_per_step / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the block-contraction join (one launch = all 8 block products of one vertex)
    join_ms = [x["ms"] for x in rec if x["stage"] == "join"]
    agg_ms = [x["ms"] for x in rec if x["stage"] == "aggregate"]
    avg_join = sum(join_ms) / max(1, len(join_ms))
    achieved = 2.0 * n * n * n / (avg_join * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "k_contract (bf16 MFMA block contraction, 8 tuples per launch)",
                "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                "avg_launch_ms": avg_join, "traffic": None}
    extra = {}
    if agg_ms:
        # aggregation: n_agg fp32 slabs read + one output written per launch (bf16 for A.B, fp32 for the result)
        byts = []
        for v in w.einsum_vertices():
            pl = r.plan(v.name)
            if pl["n_agg"] > 1:
                byts.append(pl["n_agg"] * n * n * 4 + n * n * (2 if v.dtype == "bf16" else 4))
        per = [b / (m * 1e-3) / 1e9 for b, m in zip(byts * args.steps, agg_ms)]
        avg = sum(per) / len(per)
        extra["aggregate"] = {"bound": "hbm", "achieved": avg, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": avg / PEAK_HBM_GBS,
                              "avg_launch_ms": sum(agg_ms) / len(agg_ms)}
    out = {"metric": "einsum-graph TFLOP/s (contractions), % of roofline", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{w.name}: (A.B).C, all sides {n}, bf16 in / fp32 accumulate, partitioning '{args.partitioning}' "
                                  f"({json.dumps(r.part)})"},
           "roofline": roofline, "other_kernels": extra}
    r.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
