#!/usr/bin/env python3
"""Benchmark of the tensor-relational einsum hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: tr_execute of a workload graph,
i.e. for every vertex the join kernel over all block tuples and, where a contracted label is partitioned,
the aggregation of the fp32 partial slabs.  The default workload is the matrix chain (A.B).C with
i=j=k=l=8192, bf16 storage, fp32 accumulation, first product cut (2,2,2), second cut (1,2,4) (so a
repartition of A.B sits between them).  Inputs are resident in HBM before the timed region.
Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA (datasheet)
PEAK_F32_TFLOPS = 157.3       # MI355X dense fp32 MFMA (datasheet); config 1 is the only fp32 workload
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E (datasheet)
# vector-ALU bound of the distance contractions: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3e12 fused
# multiply-adds per second (packed fp32 instructions are not used); every label combination costs one of them (or
# one maximum) plus a subtraction, which the hardware issues beside it (measured: the pair runs at the rate of the
# multiply-add alone), and is counted as three operations (subtract, multiply, add)
PEAK_ALU_TFLOPS = 256 * 4 * 16 * 2.4e9 * 3 / 1e12
DEFAULT_PART = {1: "d222", 2: "mix", 3: "batch8", 4: "heads8", 5: "k16", 6: "splitn8", 7: "d222"}
# HBM-side bytes per launch (mean over the family's launches of a step) from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this
# file, scaled by what the same counters read for the plain 1 GiB copy kernel (see profiles/); a family that is not listed
# reports null.  Keys: (workload, partitioning, kernel family).
MEASURED_TRAFFIC = {
    ("c2", "mix", "contract_mfma"): 2189732864,    # 1575 MiB fetched + 513 MiB written per launch (1575-1690 MiB fetched over the pool's boxes)
    ("c2", "mix", "aggregate"): 739217408,         # 512 MiB fetched + 193 MiB written
    ("c3", "batch8", "contract_mfma"): 481092000,  # 212 MiB fetched + 247 MiB written (mean over the step's five contractions)
    ("c3", "batch8", "map"): 83944448,             # 48 MiB fetched + 32 MiB written (mean over the ReLU and its gradient; the other maps run inside the softmax pass)
    ("c3", "batch8", "softmax_fused"): 51062784,   # 24.7 MiB fetched (logits and labels) + 24 MiB written (log-probabilities and the gradient dL)
    ("c3", "batch8", "reduce_row"): 25293930,      # 24 MiB fetched
    ("c3", "batch8", "aggregate"): 453230000,      # 384 MiB fetched + 48 MiB written (mean over the step's three aggregations)
    ("c4", "heads8", "contract_mfma"): 1280241700, # 812 MiB fetched + 409 MiB written (mean over the step's nine contractions)
    ("c4", "heads8", "softmax_fused"): 2281005450, # 1152 MiB fetched (scores + the mask rows) + 1023 MiB written
    ("c4", "heads8", "aggregate"): 1174699000,     # 1024 MiB fetched + 96 MiB written
    ("c4", "heads8", "map"): 549389600,            # 352 MiB fetched + 172 MiB written
    ("c5", "k16", "contract_mfma"): 31395302400,   # 13556 MiB fetched (L2 misses; the re-reads of X are served by the Infinity Cache) + 16385 MiB written
    ("c5", "k16", "aggregate"): 18253883392,       # 16384 MiB fetched + 1024 MiB written
}


def prod(xs):
    p = 1
    for x in xs:
        p *= int(x)
    return p


def cpu_baseline(w, dev, budget_s=15.0):
    """Times the oracle as it stands on a bounded sample: R rows of the first contraction at full reduction length."""
    import numpy as np
    import torch
    from oracle.einsum_ref import einsum_ref
    from synth_inputs.workloads import parse_spec
    v = next(v for v in w.einsum_vertices() if v.oplus != "none" and len(v.inputs) == 2
             and all(w.vertex(i).is_input for i in v.inputs))
    per_pair = 2.0 if v.otimes == "mul" else 3.0

    def host(t):
        t = t.detach().contiguous().cpu()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    X, Y = host(dev[v.inputs[0]]), host(dev[v.inputs[1]])
    lX, lY, lZ = parse_spec(v.spec)
    per_row = per_pair * prod(X.shape[1:]) * prod(n for l, n in zip(lY, Y.shape) if l not in lX)

    def run(rows):
        t0 = time.perf_counter()
        einsum_ref(v.spec, X[:rows], Y, otimes=v.otimes, oplus=v.oplus, alpha=v.alpha, out_dtype=v.dtype,
                   x_dtype=w.vertex(v.inputs[0]).dtype, y_dtype=w.vertex(v.inputs[1]).dtype)
        return time.perf_counter() - t0

    r0 = max(1, min(X.shape[0], 4))
    t = run(r0)
    rows = int(max(r0, min(X.shape[0], r0 * budget_s / max(t, 1e-3))))
    t = run(rows)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    from oracle import build as oracle_build
    return {"value": per_row * rows / t / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "build": "gcc " + " ".join(oracle_build.FLAGS) + " (oracle/einsum_ref.c as it stands; x86-64-v2 because the library is built on another machine than it is timed on)",
            "sample": f"vertex {v.name} '{v.spec}': {rows} of {X.shape[0]} outer rows at full reduction length "
                      f"(einsum_ref loop nest, double accumulation), {t:.1f} s"}


def ceilings():
    """Measured ceilings of this machine: register-resident bf16 MFMA loop and a plain copy."""
    import torch
    import paper_2410_02682_amd as E
    s = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(16, device="cuda")
    out = {}
    for wps in (1, 2):
        E.eg_ceiling_mfma_bf16(sink.data_ptr(), 256, wps, 2000, s)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fl = E.eg_ceiling_mfma_bf16(sink.data_ptr(), 256, wps, 20000, s)
        b.record()
        torch.cuda.synchronize()
        out[f"mfma_bf16_{wps}_wave_per_simd_tflops"] = fl / a.elapsed_time(b) / 1e9
    # the same loop on pseudo-random operands: the chip's clock under the matrix pipes depends on the operand bits
    E.eg_ceiling_mfma_bf16_random(sink.data_ptr(), 256, 1000, s)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    fl = E.eg_ceiling_mfma_bf16_random(sink.data_ptr(), 256, 10000, s)
    b.record()
    torch.cuda.synchronize()
    out["mfma_bf16_random_operands_tflops"] = fl / a.elapsed_time(b) / 1e9
    E.eg_ceiling_valu_f32(sink.data_ptr(), 256, 2, 500, s)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    pairs = E.eg_ceiling_valu_f32(sink.data_ptr(), 256, 2, 10000, s)
    b.record()
    torch.cuda.synchronize()
    out["valu_f32_sub_fma_pairs_as_tflops"] = 3.0 * pairs / a.elapsed_time(b) / 1e9
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    E.eg_ceiling_copy(dst.data_ptr(), src.data_ptr(), n, s)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        E.eg_ceiling_copy(dst.data_ptr(), src.data_ptr(), n, s)
    b.record()
    torch.cuda.synchronize()
    out["copy_read_plus_write_gbs"] = 2 * n * 5 / a.elapsed_time(b) / 1e6
    del src, dst
    # read-mostly streams with the traffic shape of an aggregation of 2, 8 and 16 partial slabs (256 MiB pieces)
    piece = 1 << 28
    src = torch.empty(16 * piece, dtype=torch.uint8, device="cuda")
    dst = torch.empty(piece, dtype=torch.uint8, device="cuda")
    for streams in (2, 8, 16):
        E.eg_ceiling_read(dst.data_ptr(), src.data_ptr(), streams, piece, s)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            E.eg_ceiling_read(dst.data_ptr(), src.data_ptr(), streams, piece, s)
        b.record()
        torch.cuda.synchronize()
        out[f"read_{streams}_pieces_write_1_gbs"] = (streams + 1) * piece * 5 / a.elapsed_time(b) / 1e6
    return out


KERNEL_TEXT = {"contract_mfma": "k_contract_dma / k_contract (block contraction on MFMA, all tuples of a vertex per launch)",
               "aggregate": "k_aggregate_patches (tile-ordered partial slabs) / k_aggregate_vec4 (dense ones)", "map": "k_map", "reduce_row": "k_reduce_row", "generic": "k_generic",
               "contract_alu": "k_contract_alu (contraction-shaped vertex with another scalar function, vector ALU)",
               "softmax_fused": "k_softmax_rows / k_softmax_rows_bf16 (softmax chain, the sum in front and the element-wise vertices behind it in one pass per row)",
               "attention_fused": "k_attention (scores contraction, softmax chain and weighted sum in one pass; alternative, off by default)"}


def measure(config, pname, steps, warmup, fuse_aggregation=False, contract=None, fuse_attention=False, dense_partials=False):
    """Times `steps` passes of one workload under one partitioning: (per-step ms, per-family kernel records, flops per step,
    workload description, device inputs, the workload)."""
    import torch
    import paper_2410_02682_amd as E
    from paper_2410_02682_amd.runner import GraphRunner
    from synth_inputs import build_config, prng_torch

    w = build_config(config)
    dev = {v.name: prng_torch.make_tensor(v.recipe, v.bound, v.dtype, w.seed, w.tensor_id(v.name)) for v in w.vertices if v.is_input}
    r = GraphRunner(w, pname, contract=contract, fuse_aggregation=True if fuse_aggregation else None, fuse_attention=True if fuse_attention else None, tiled_partials=False if dense_partials else None)
    r.bind(dev)
    stream = torch.cuda.current_stream()
    # A working set that the 256 MiB Infinity Cache could hold between steps is rotated over three copies (inputs,
    # workspace and outputs), so that no step finds its operands left there by the previous one.
    esz = {"f32": 4, "bf16": 2}
    working_set = sum(prod(v.bound) * esz[v.dtype] for v in w.vertices if v.is_input) + r.workspace_bytes \
        + sum(r.output(n).numel() * r.output(n).element_size() for n in r.out_names)
    runners = [r]
    if working_set < (512 << 20):
        for _ in range(2):
            r2 = GraphRunner(w, pname, contract=contract, fuse_aggregation=True if fuse_aggregation else None, fuse_attention=True if fuse_attention else None, tiled_partials=False if dense_partials else None)
            r2.bind({k: t.clone() for k, t in dev.items()})
            runners.append(r2)
    for i in range(warmup * len(runners)):
        runners[i % len(runners)].run(stream)
    torch.cuda.synchronize()

    # per-vertex accounting: flops of contractions, algorithmic bytes of every launch
    acct = {}
    for v in w.einsum_vertices():
        pl = r.plan(v.name)
        nz = prod(pl["bound_z"])
        in_bytes = sum(prod(w.vertex(i).bound if w.vertex(i).is_input else r.plan(i)["bound_z"]) * esz[w.vertex(i).dtype] for i in v.inputs)
        acct[r.vid[v.name]] = {
            "name": v.name, "kind": pl["kernel"], "nz": nz, "esz": esz[v.dtype], "in_bytes": in_bytes,
            # a multiply-add per label combination on the matrix pipes; subtract, square (or magnitude), add (or max) on the vector ALU
            "flops": {"contract_mfma": 2.0, "contract_alu": 3.0}.get(pl["kernel"], 0.0) * prod(pl["bound"]),
            # a fused softmax pass is credited its own minimal traffic: one tensor of the result's shape in, the result out
            "fused_bytes": nz * (esz[v.dtype] + esz[w.vertex(v.inputs[0]).dtype]),
        }
    # the event log is sized generously (the execution adds aggregation launches of its own to vertices whose reduction
    # it cuts further, and runs a fused softmax chain as one launch); what was recorded is read back, never assumed
    capacity = 4 * len(acct) * steps + 16
    for q in runners:
        E.tr_profile_enable(q.g, capacity)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        runners[i % len(runners)].run(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    rec = [x for q in runners for x in E.tr_profile_read(q.g)]        # vertex ids are the same in every copy
    assert len(rec) % steps == 0 and all(len(E.tr_profile_read(q.g)) < capacity for q in runners), "launch log overflow"
    ms_per_step = (t1 - t0) * 1e3 / steps
    flops_per_step = sum(a["flops"] for a in acct.values())

    # A fused softmax pass is recorded at its division; the vertices it absorbed (the chain, a sum in front, element-wise
    # vertices behind) have no launch of their own.  Its algorithmic bytes: what those vertices read from outside their
    # set + what of theirs anything outside the set reads (or the caller asked for), each tensor once.  (With the one-pass
    # attention in the same graph the absorbed sets cannot be told apart this way and the chain alone is credited.)
    launched = {x["vertex"] for x in rec}
    fused_pass_bytes = None
    if any(x["kernel"] == "softmax_fused" for x in rec) and not any(x["kernel"] == "attention_fused" for x in rec):
        absorbed = {v.name for v in w.einsum_vertices() if r.vid[v.name] not in launched}
        absorbed |= {a["name"] for vid_, a in acct.items() if any(x["vertex"] == vid_ and x["kernel"] == "softmax_fused" for x in rec)}
        size = lambda name: prod(w.vertex(name).bound if w.vertex(name).is_input else r.plan(name)["bound_z"]) * esz[w.vertex(name).dtype]
        reads = {i for v in w.einsum_vertices() if v.name in absorbed for i in v.inputs if i not in absorbed}
        writes = {n for n in absorbed if n in w.outputs or any(n in v.inputs for v in w.einsum_vertices() if v.name not in absorbed)}
        fused_pass_bytes = sum(size(n) for n in reads | writes)
        n_fused_per_step = sum(1 for x in rec if x["kernel"] == "softmax_fused") / steps
    # aggregate the recorded launches by kernel family; bytes as the execution really ran them: a join launch reads its
    # inputs and writes `slabs` fp32 partial slabs (or its tensor), an aggregation reads `slabs` slabs and writes the tensor
    fam = {}
    for x in rec:
        a = acct[x["vertex"]]
        key = "aggregate" if x["stage"] == "aggregate" else ("softmax_fused" if x["kernel"] == "softmax_fused" else x["kernel"])
        f = fam.setdefault(key, {"ms": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0, "each": []})
        f["each"].append(x["ms"])
        f["ms"] += x["ms"]
        f["launches"] += 1
        if x["stage"] == "aggregate":
            f["bytes"] += x["slabs"] * a["nz"] * 4 + a["nz"] * a["esz"]
        elif key == "softmax_fused":
            f["bytes"] += fused_pass_bytes / n_fused_per_step if fused_pass_bytes is not None else a["fused_bytes"]
        elif key == "attention_fused":
            # recorded at the second contraction; the first one runs over the same label combinations, so the launch
            # does twice that vertex's operations (no key block is skipped under a causal mask)
            f["flops"] += 2 * a["flops"]
        else:
            f["flops"] += a["flops"]
            f["bytes"] += a["in_bytes"] + (x["slabs"] * a["nz"] * 4 if x["slabs"] else a["nz"] * a["esz"])
    kernels = {}
    for key, f in fam.items():
        each = sorted(f["each"])
        k = {"launches_per_step": f["launches"] / steps, "avg_launch_ms": f["ms"] / f["launches"],
             "median_launch_ms": each[len(each) // 2], "min_launch_ms": each[0],
             "share_of_step": f["ms"] / steps / ms_per_step}
        if key in ("contract_mfma", "attention_fused"):
            k.update({"bound": "mfma", "achieved": f["flops"] / (f["ms"] * 1e-3) / 1e12,
                      "peak": PEAK_F32_TFLOPS if config == 1 else PEAK_BF16_TFLOPS, "unit": "TFLOP/s"})
        elif key == "contract_alu":
            k.update({"bound": "alu", "achieved": f["flops"] / (f["ms"] * 1e-3) / 1e12, "peak": PEAK_ALU_TFLOPS, "unit": "TFLOP/s"})
        else:
            k.update({"bound": "hbm", "achieved": f["bytes"] / (f["ms"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"})
        k["frac"] = k["achieved"] / k["peak"]
        t = MEASURED_TRAFFIC.get((f"c{config}", pname, key))
        k["traffic"] = t
        kernels[key] = k
    # The same steps once more as replays of captured HIP graphs (one graph per buffer set; tr_execute only enqueues
    # kernels, so a caller may capture it): what launch gaps cost.  Reported beside the eager figure, never instead of it.
    graph_ms = None
    try:
        for q in runners:
            E.tr_profile_enable(q.g, 0)
        side = torch.cuda.Stream()
        graphs = []
        with torch.cuda.stream(side):
            for q in runners:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    q.run(torch.cuda.current_stream())
                graphs.append(g)
        torch.cuda.synchronize()
        for i in range(max(warmup, 1) * len(graphs)):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for i in range(steps):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) * 1e3 / steps
        del graphs
    except Exception as e:                               # the eager figures above stand on their own
        print(f"bench.py: HIP graph replay not measured ({e})", file=sys.stderr)
    desc = f"{w.name} dims {json.dumps(w.dims)}, partitioning '{pname}': {json.dumps(r.part)}" \
        + (" [alternative method: aggregation inside the contraction kernels]" if fuse_aggregation else "") \
        + (" [alternative: attention as one pass]" if fuse_attention else "") \
        + (" [comparison: dense partial slabs]" if dense_partials else "")
    n_sets = len(runners)
    for q in runners[1:]:
        q.close()
    r.close()
    return ms_per_step, kernels, flops_per_step, desc, dev, w, (n_sets, graph_ms)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5, 6, 7], help="workload (2 = the matrix chain the metric is quoted on)")
    ap.add_argument("--partitioning", default=None)
    ap.add_argument("--fuse-aggregation", action="store_true",
                    help="alternative method, reported separately: contractions reduce over partitioned contracted labels inside the kernel (no partial slabs, no aggregation launch)")
    ap.add_argument("--fuse-attention", action="store_true",
                    help="alternative, reported separately: attention groups (scores contraction, softmax chain, weighted sum) run as one kernel")
    ap.add_argument("--dense-partials", action="store_true",
                    help="for comparisons: partial slabs as dense row-major tensors instead of in the contraction kernel's tile order")
    ap.add_argument("--contract-tile", default=None, help="for comparisons: output tile of the block-contraction kernel, e.g. 256x256, 256x128, 128 (default: the library chooses)")
    ap.add_argument("--contract-waves", type=int, default=0, help="for comparisons: 4 or 8 waves per workgroup of the 256 x 256 tile")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the short runs of configs 3, 4 and 5 that follow the headline workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    pname = args.partitioning or DEFAULT_PART[args.config]
    contract = None
    if args.contract_tile:
        t = [int(x) for x in args.contract_tile.split("x")]
        contract = dict(tile=(t[0], t[-1]), waves=args.contract_waves)
    ms_per_step, kernels, flops_per_step, desc, dev, w, (n_sets, graph_ms) = measure(args.config, pname, args.steps, args.warmup, args.fuse_aggregation, contract, args.fuse_attention, args.dense_partials)
    value = flops_per_step / (ms_per_step * 1e-3) / 1e12

    dom = "contract_mfma" if "contract_mfma" in kernels else max(kernels, key=lambda k: kernels[k]["share_of_step"])
    if args.config == 7:
        dom = "contract_alu"
    roofline = dict(kernels[dom])
    roofline["kernel"] = KERNEL_TEXT[dom]
    out = {"metric": "einsum-graph TFLOP/s (contractions) + GB/s (maps/aggregations), % of roofline", "value": value,
           "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32" if args.config == 1 else "bf16", "data": "synthetic",
           "config": {"workload": desc},
           "roofline": roofline, "kernels": kernels, "buffer_sets": n_sets, "hip_graph_replay_ms_per_step": graph_ms}
    if not args.no_ceilings:
        try:
            out["measured_ceilings"] = ceilings()
        except Exception as e:          # context only: the line above does not depend on it
            out["measured_ceilings"] = {"error": f"{type(e).__name__}: {e}"}
        if dom == "contract_mfma" and args.config != 1 and "mfma_bf16_random_operands_tflops" in out["measured_ceilings"]:
            # the rate a contraction on real data can be held against on this machine: the register-resident MFMA loop on random operands
            out["roofline"]["frac_of_measured_mfma_ceiling"] = roofline["achieved"] / out["measured_ceilings"]["mfma_bf16_random_operands_tflops"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, dev)
    del dev
    torch.cuda.empty_cache()
    if not args.no_other_workloads and args.config == 2 and not args.fuse_aggregation and not args.fuse_attention and not args.dense_partials and contract is None:
        # the other full-size workloads, a few steps each, so that their kernel families are measured in the same run
        others = {}
        for c, alt in ((3, False), (4, False), (5, False), (4, True)):
            key = f"c{c}" + ("_attention_as_one_pass" if alt else "")
            try:
                ms, ks, fl, d, dv, _, (_, gms) = measure(c, DEFAULT_PART[c], 12 if c == 3 else 5, 3 if c == 3 else 2, fuse_attention=alt)   # (config 3's step is a millisecond)
            except Exception as e:      # the headline line must not depend on these legs (they need up to 40 GiB of device memory)
                others[key] = {"error": f"{type(e).__name__}: {e}"}
                torch.cuda.empty_cache()
                continue
            del dv
            torch.cuda.empty_cache()
            others[key] = {"workload": d, "ms_per_step": ms, "hip_graph_replay_ms_per_step": gms, "contraction_tflops_per_step": fl / (ms * 1e-3) / 1e12,
                               "kernels": {k: {f: v[f] for f in ("launches_per_step", "avg_launch_ms", "bound", "achieved", "peak", "unit", "frac", "traffic")}
                                           for k, v in ks.items()}}
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
