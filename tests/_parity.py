"""Shared helpers of the GPU parity tests: tolerance rule and ad-hoc one-vertex workloads."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from synth_inputs.prng import HostTensor
from synth_inputs.workloads import Vertex, Workload

RTOL_F32 = 1e-5      # fp32 storage, fp32 accumulation, exact inputs
RTOL_BF16 = 2e-2     # bf16 outputs with fp32 accumulation, or anything downstream of a bf16-rounded intermediate


def violations(got: np.ndarray, ref: np.ndarray, rtol: float):
    """Element-wise |g - r| <= rtol*|r| + rtol*rms(r); non-finite reference entries must match exactly.

    Returns (number of violating elements, worst ratio of error to allowance)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    assert got.shape == ref.shape
    fin = np.isfinite(ref)
    bad = int(np.sum(got[~fin] != ref[~fin]))
    if fin.any():
        r, g = ref[fin], got[fin]
        rms = float(np.sqrt(np.mean(r * r)))
        allow = rtol * np.abs(r) + rtol * rms + 1e-300
        err = np.abs(g - r)
        err = np.where(np.isfinite(err), err, np.inf)
        ratio = err / allow
        bad += int(np.sum(ratio > 1.0))
        worst = float(ratio.max())
    else:
        worst = 0.0
    return bad, worst


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
