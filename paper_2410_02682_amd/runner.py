"""Binds a workload description (synth_inputs.workloads.Workload) to the C ABI: marshalling only.

Builds the library's EinGraph from the vertex records, annotates it with one named set of
partitioning vectors, views torch device tensors as tensor relations and calls tr_execute.
torch is used for device memory and the stream handle only.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional

import numpy as np
import torch

from synth_inputs.prng import HostTensor
from synth_inputs.workloads import Workload, d_vector, parse_spec
from . import api

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def to_device(t: HostTensor, device="cuda") -> torch.Tensor:
    if t.dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(t.data)).to(device)
    return torch.from_numpy(np.ascontiguousarray(t.data).view(np.int16)).to(device).view(torch.bfloat16)


def to_host(x: torch.Tensor) -> HostTensor:
    x = x.detach().contiguous().cpu()
    if x.dtype == torch.float32:
        return HostTensor(x.numpy().copy(), "f32")
    return HostTensor(x.view(torch.int16).numpy().view(np.uint16).copy(), "bf16")


class GraphRunner:
    def __init__(self, w: Workload, partitioning: str, outputs: Optional[Iterable[str]] = None, device="cuda",
                 contract: Optional[dict] = None, fuse: Optional[bool] = None, fuse_aggregation: Optional[bool] = None,
                 fuse_attention: Optional[bool] = None, tiled_partials: Optional[bool] = None):
        """contract: arguments of tr_set_contract_variant (kernel / tile / waves); fuse, fuse_aggregation, fuse_attention:
        arguments of tr_set_fusion, tr_set_fused_aggregation and tr_set_fused_attention; tiled_partials: of
        tr_set_tiled_partials.  None leaves the library's defaults."""
        self.w = w
        self.device = device
        self.g = api.einsum_graph_create()
        if contract:
            api.tr_set_contract_variant(self.g, **contract)
        if fuse is not None:
            api.tr_set_fusion(self.g, fuse)
        if fuse_aggregation is not None:
            api.tr_set_fused_aggregation(self.g, fuse_aggregation)
        if fuse_attention is not None:
            api.tr_set_fused_attention(self.g, fuse_attention)
        if tiled_partials is not None:
            api.tr_set_tiled_partials(self.g, tiled_partials)
        self.vid: Dict[str, int] = {}
        # "eindecomp:<p>": let the library choose the partitioning vectors (p join results per vertex)
        planned = partitioning.startswith("eindecomp:")
        self.part = {} if planned else w.partitionings[partitioning]
        self.out_names = list(outputs) if outputs is not None else list(w.outputs)
        for v in w.vertices:
            if v.is_input:
                self.vid[v.name] = api.einsum_graph_add_input(self.g, v.bound, v.dtype)
            else:
                self.vid[v.name] = api.einsum_graph_add_einsum(self.g, v.spec, v.otimes, v.oplus, v.alpha,
                                                               [self.vid[n] for n in v.inputs], v.dtype)
                api.einsum_graph_set_partition(self.g, self.vid[v.name], d_vector(v.spec, self.part.get(v.name, {})))
        self.plan_cost = None
        if planned:
            self.plan_cost, self.plan_exact = api.eindecomp_plan(self.g, int(partitioning.split(":")[1]))
            for v in w.einsum_vertices():
                pl = api.einsum_graph_plan(self.g, self.vid[v.name])
                self.part[v.name] = {l: int(x) for l, x in zip(pl["labels"], pl["d"]) if x > 1}
        for n in self.out_names:
            api.einsum_graph_mark_output(self.g, self.vid[n])
        self.rel_in, self.rel_out = [], []
        self.tensors: Dict[str, torch.Tensor] = {}
        self.workspace = None

    def plan(self, name: str) -> dict:
        return api.einsum_graph_plan(self.g, self.vid[name])

    def _input_partition(self, name: str):
        """Inputs are pre-partitioned the way their first consumer joins them (Section 8.2: inputs cost nothing)."""
        for v in self.w.einsum_vertices():
            for pos, n in enumerate(v.inputs):
                if n == name:
                    lX, lY, _ = parse_spec(v.spec)
                    labs = lX if pos == 0 else lY
                    part = self.part.get(v.name, {})
                    return [int(part.get(l, 1)) for l in labs]
        return [1] * len(self.w.vertex(name).bound)

    def bind(self, inputs: Dict[str, torch.Tensor], outputs: Optional[Dict[str, torch.Tensor]] = None, workspace: bool = True):
        """Views the given device tensors as tensor relations.  Any strided view will do (a relation is a base pointer,
        bounds and element strides); outputs not given are allocated dense.  workspace=False: no workspace is
        allocated (for run_static, which uses the library's own)."""
        self.release_relations()
        for v in self.w.vertices:
            if v.is_input:
                t = inputs[v.name]
                assert tuple(t.shape) == tuple(v.bound) and t.dtype == TORCH_DTYPE[v.dtype]
                self.tensors[v.name] = t
                self.rel_in.append(api.tensor_partition(t.data_ptr(), v.dtype, v.bound, self._input_partition(v.name),
                                                        strides=None if t.is_contiguous() else list(t.stride())))
        for n in self.out_names:
            v = self.w.vertex(n)
            pl = self.plan(n)
            if outputs is not None and n in outputs:
                t = outputs[n]
                assert tuple(t.shape) == tuple(pl["bound_z"]) and t.dtype == TORCH_DTYPE[v.dtype]
            else:
                t = torch.empty(tuple(pl["bound_z"]), dtype=TORCH_DTYPE[v.dtype], device=self.device)
            self.tensors[n] = t
            self.rel_out.append(api.tensor_partition(t.data_ptr(), v.dtype, pl["bound_z"], pl["d_z"],
                                                     strides=None if t.is_contiguous() else list(t.stride())))
        nbytes = api.tr_workspace_bytes(self.g)
        self.workspace_bytes = nbytes
        if workspace:
            self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
            assert self.workspace.data_ptr() % 256 == 0
        return self

    def run(self, stream: Optional[torch.cuda.Stream] = None):
        s = stream if stream is not None else torch.cuda.current_stream()
        api.tr_execute(self.g, self.rel_in, self.rel_out, self.workspace.data_ptr(), self.workspace.numel(), s.cuda_stream)

    def run_static(self, stream: Optional[torch.cuda.Stream] = None):
        """tr_execute_static: the same pass with the library's static workspace (nothing is allocated)."""
        s = stream if stream is not None else torch.cuda.current_stream()
        api.tr_execute_static(self.g, self.rel_in, self.rel_out, s.cuda_stream)

    def output(self, name: str) -> torch.Tensor:
        return self.tensors[name]

    def release_relations(self):
        for r in self.rel_in + self.rel_out:
            api.tensor_relation_destroy(r)
        self.rel_in, self.rel_out = [], []

    def close(self):
        self.release_relations()
        if self.g is not None:
            api.einsum_graph_destroy(self.g)
            self.g = None
