"""Vertex-by-vertex oracle evaluation of a workload graph.  TEST INFRASTRUCTURE ONLY.

An EinGraph (Section 5 of the paper) is evaluated in the order its vertices
are listed (a topological order); each einsum vertex is one call of the
loop-nest oracle on the stored values of its inputs, rounded once to the
vertex's storage dtype, so a bf16 intermediate is rounded at the same place
as in the HIP graph.  The result does not depend on any partitioning vector.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional

import numpy as np

from synth_inputs.prng import HostTensor, make_tensor
from synth_inputs.workloads import Workload
from .einsum_ref import einsum_ref


def to_storage(values_f64: np.ndarray, dtype: str) -> HostTensor:
    """Values already rounded to dtype (as float64) -> storage array."""
    shape = np.shape(values_f64)
    f = np.ascontiguousarray(np.asarray(values_f64, dtype=np.float64).astype(np.float32)).reshape(shape)
    if dtype == "f32":
        return HostTensor(f, "f32")
    bits = (f.reshape(-1).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return HostTensor(bits.reshape(shape), "bf16")


def make_inputs(w: Workload) -> Dict[str, HostTensor]:
    return {v.name: make_tensor(v.recipe, v.bound, v.dtype, w.seed, w.tensor_id(v.name))
            for v in w.vertices if v.is_input}


def run_graph(w: Workload, inputs: Dict[str, HostTensor], keep: Optional[Iterable[str]] = None) -> Dict[str, HostTensor]:
    """Evaluate every vertex; returns all tensors (or only `keep` plus inputs)."""
    env: Dict[str, HostTensor] = dict(inputs)
    for v in w.vertices:
        if v.is_input:
            continue
        X = env[v.inputs[0]]
        Y = env[v.inputs[1]] if len(v.inputs) > 1 else None
        z = einsum_ref(v.spec, X.data, None if Y is None else Y.data,
                       otimes=v.otimes, oplus=v.oplus, alpha=v.alpha, out_dtype=v.dtype,
                       x_dtype=X.dtype, y_dtype=None if Y is None else Y.dtype)
        env[v.name] = to_storage(z, v.dtype)
    if keep is not None:
        keep = set(keep)
        return {k: t for k, t in env.items() if k in keep}
    return env
