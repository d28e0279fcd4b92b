"""Shared helpers of the GPU parity tests: tolerance rule and ad-hoc one-vertex workloads."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from synth_inputs.prng import HostTensor
from synth_inputs.workloads import Vertex, Workload

RTOL_F32 = 1e-5      # fp32 storage, fp32 accumulation, exact inputs
RTOL_BF16 = 2e-2     # bf16 outputs with fp32 accumulation, or anything downstream of a bf16-rounded intermediate


EPS_F32 = 2.0 ** -24


def violations(got: np.ndarray, ref: np.ndarray, rtol: float, magnitude: Optional[np.ndarray] = None, report: Optional[dict] = None):
    """Element-wise |g - r| <= rtol*|r| + rtol*rms(r); non-finite reference entries must match exactly.

    magnitude (optional, same shape): the sum of the absolute values of the terms behind every element, as
    `magnitudes` computes it.  fp32 summation, compensated or not, errs by a few 2^-24 of THAT sum, whatever
    is left after cancellation (compensated summation: 2 * 2^-24, plus one rounding of each stored operand and
    of each partial block).  An element that fails the plain rule is accepted if it is within the plain allowance
    plus 4 * 2^-24 * magnitude; how many elements needed that is counted in report["leaned_on_magnitude"], so a
    change that starts to lean on the allowance shows.  For K products of random sign the sum of absolute values
    is about 0.6 * sqrt(K) times the result, so at K = 1000 the extra term is half of rtol = 1e-5.

    report (optional dict) also receives "strict_worst": the largest plain relative error |g - r| / |r| over the
    elements with |r| >= rms(r), i.e. the figure the stated targets (1e-5 for fp32 results, 2e-2 for bf16 ones)
    are about, free of the rms term and of the magnitude allowance.

    Returns (number of violating elements, worst ratio of error to allowance)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    assert got.shape == ref.shape
    fin = np.isfinite(ref)
    bad = int(np.sum(got[~fin] != ref[~fin]))
    leaned, strict = 0, 0.0
    if fin.any():
        r, g = ref[fin], got[fin]
        rms = float(np.sqrt(np.mean(r * r)))
        allow = rtol * np.abs(r) + rtol * rms + 1e-300
        err = np.abs(g - r)
        err = np.where(np.isfinite(err), err, np.inf)
        ratio = err / allow
        if magnitude is not None:
            fails = ratio > 1.0
            if fails.any():
                m = np.asarray(magnitude, dtype=np.float64).ravel()[fin][fails]
                wide = allow[fails] + 4 * EPS_F32 * np.where(np.isfinite(m), np.abs(m), 0.0)
                ratio[fails] = err[fails] / wide
                leaned = int(np.sum(ratio[fails] <= 1.0))
        bad += int(np.sum(ratio > 1.0))
        worst = float(ratio.max())
        big = np.abs(r) >= rms
        if big.any() and rms > 0:
            strict = float(np.max(err[big] / np.abs(r[big])))
    else:
        worst = 0.0
    if report is not None:
        report["leaned_on_magnitude"] = report.get("leaned_on_magnitude", 0) + leaned
        report["strict_worst"] = max(report.get("strict_worst", 0.0), strict)
    return bad, worst


def tile_of(text: str):
    """'256x128' -> (256, 128), '128' -> (128, 128), '' -> 0: the tile argument of tr_set_contract_variant."""
    if not text:
        return 0
    parts = [int(t) for t in str(text).split("x")]
    return (parts[0], parts[-1])


def tainted_by_bf16(w: Workload) -> Dict[str, bool]:
    """A vertex carries bf16 rounding error if it or any computed ancestor is stored in bf16."""
    t: Dict[str, bool] = {}
    for v in w.vertices:
        if v.is_input:
            t[v.name] = False
        else:
            t[v.name] = v.dtype == "bf16" or any(t[i] for i in v.inputs)
    return t


def rtol_for(w: Workload, name: str) -> float:
    return RTOL_BF16 if tainted_by_bf16(w)[name] else RTOL_F32


def single_vertex(spec: str, x: HostTensor, y: Optional[HostTensor], out_dtype: str, otimes="mul", oplus="sum",
                  alpha=1.0, parts=None) -> Workload:
    vs = [Vertex("X", x.dtype, bound=tuple(x.shape))]
    ins = ["X"]
    if y is not None:
        vs.append(Vertex("Y", y.dtype, bound=tuple(y.shape)))
        ins.append("Y")
    vs.append(Vertex("Z", out_dtype, spec=spec, otimes=otimes, oplus=oplus, alpha=alpha, inputs=tuple(ins)))
    return Workload("adhoc", 0, vs, ["Z"], {k: {"Z": v} for k, v in (parts or {"whole": {}}).items()})



def magnitudes(w: Workload, inputs: Dict[str, HostTensor]) -> Dict[str, HostTensor]:
    """Every vertex of the graph evaluated by the oracle on the absolute values of the inputs, with differences
    turned into sums and scale factors into their absolute values: for sums of products (and of anything built
    from them) that is the sum of the absolute values of the terms, the quantity rounding errors of a
    floating-point sum are proportional to.  Scalar functions that cannot cancel are evaluated as they are."""
    from dataclasses import replace
    from oracle.graph_ref import run_graph

    def plain(v: Vertex) -> Vertex:
        if v.is_input:
            return v
        otimes, alpha = v.otimes, abs(v.alpha)
        if otimes == "sub":
            otimes, alpha = "add", 1.0
        return replace(v, otimes=otimes, alpha=alpha)

    wm = Workload(w.name + "_magnitude", w.seed, [plain(v) for v in w.vertices], [v.name for v in w.einsum_vertices()])

    def absolute(t: HostTensor) -> HostTensor:
        return HostTensor(t.data & np.uint16(0x7FFF), "bf16") if t.dtype == "bf16" else HostTensor(np.abs(t.data), "f32")

    return run_graph(wm, {k: absolute(t) for k, t in inputs.items()})
