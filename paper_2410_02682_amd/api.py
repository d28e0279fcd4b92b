"""Thin Python binding over the C ABI (include/eindecomp.h): argument marshalling only.

Every step of the path runs inside libeindecomp.so.  The functions below carry the
names of the C entry points; `Graph` and `Relation` only keep handles alive and
turn Python lists into C arrays.  Device memory is handed over as raw pointers
(e.g. torch.Tensor.data_ptr()), streams as raw hipStream_t handles.
"""
from __future__ import annotations

import ctypes
from typing import List, Optional, Sequence, Tuple

from . import _lib
from ._lib import PlanView

DTYPE = {"f32": 0, "bf16": 1}
OPLUS = {"none": 0, "sum": 1, "max": 2}
OTIMES = {"mul": 0, "add": 1, "sub": 2, "div": 3, "sqdiff": 4, "absdiff": 5, "exp_sub": 6, "relu_grad": 7,
          "silu_mul": 8, "ident": 32, "scale": 33, "relu": 34, "exp": 35, "log": 36}
KERNEL_NAMES = {0: "none", 1: "contract_mfma", 2: "map", 3: "reduce_row", 4: "generic", 5: "contract_alu", 6: "softmax_fused", 7: "attention_fused", 8: "aggregate_tiles"}


class EgError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"eindecomp error {code}: {msg}")
        self.code = code


def _check(rc: int) -> int:
    if rc < 0:
        raise EgError(rc, _lib.load().eg_last_error().decode())
    return rc


def _i64(v: Sequence[int]):
    return (ctypes.c_int64 * max(1, len(v)))(*[int(x) for x in v])


def _i32(v: Sequence[int]):
    return (ctypes.c_int32 * max(1, len(v)))(*[int(x) for x in v])


# ---- C entry points, same names ---------------------------------------------------------------
def einsum_graph_create() -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    _check(_lib.load().einsum_graph_create(ctypes.byref(h)))
    return h


def einsum_graph_add_input(g, bound: Sequence[int], dtype: str) -> int:
    v = ctypes.c_int()
    _check(_lib.load().einsum_graph_add_input(g, len(bound), _i64(bound), DTYPE[dtype], ctypes.byref(v)))
    return v.value


def einsum_graph_add_einsum(g, spec: str, otimes: str, oplus: str, alpha: float, inputs: Sequence[int], out_dtype: str) -> int:
    v = ctypes.c_int()
    arr = (ctypes.c_int * max(1, len(inputs)))(*inputs)
    _check(_lib.load().einsum_graph_add_einsum(g, spec.encode(), OTIMES[otimes], OPLUS[oplus], float(alpha), arr,
                                               len(inputs), DTYPE[out_dtype], ctypes.byref(v)))
    return v.value


def einsum_graph_set_partition(g, vertex: int, d: Sequence[int]) -> None:
    _check(_lib.load().einsum_graph_set_partition(g, vertex, _i32(d), len(d)))


def einsum_graph_mark_output(g, vertex: int) -> None:
    _check(_lib.load().einsum_graph_mark_output(g, vertex))


def einsum_graph_plan(g, vertex: int) -> dict:
    pv = PlanView()
    _check(_lib.load().einsum_graph_plan(g, vertex, ctypes.byref(pv)))
    n, nl = pv.n_tuples, pv.n_labels
    rx, ry, rz = pv.rank_x, pv.rank_y, pv.rank_z

    def tab(ptr, cols):
        return [tuple(ptr[t * cols + c] for c in range(cols)) for t in range(n)]

    return dict(
        labels=[pv.labels[i:i + 1].decode() for i in range(nl)], bound=list(pv.bound[:nl]), d=list(pv.d[:nl]),
        d_x=list(pv.d_x[:rx]), d_y=list(pv.d_y[:ry]), d_z=list(pv.d_z[:rz]), bound_z=list(pv.bound_z[:rz]),
        block_x=list(pv.block_x[:rx]), block_y=list(pv.block_y[:ry]), block_z=list(pv.block_z[:rz]),
        n_tuples=n, n_agg=pv.n_agg, n_groups=pv.n_groups, kernel=KERNEL_NAMES[pv.kernel],
        repart_x=pv.repart_x, repart_y=pv.repart_y,
        key=tab(pv.key, nl), key_x=tab(pv.key_x, rx), key_y=tab(pv.key_y, ry), key_z=tab(pv.key_z, rz),
        agg_idx=[pv.agg_idx[t] for t in range(n)], group=[pv.group[t] for t in range(n)],
        off_x=[pv.off_x[t] for t in range(n)], off_y=[pv.off_y[t] for t in range(n)], off_z=[pv.off_z[t] for t in range(n)],
    )


def einsum_graph_destroy(g) -> None:
    _lib.load().einsum_graph_destroy(g)


def tensor_partition(dev_ptr: int, dtype: str, bound: Sequence[int], d: Sequence[int], strides: Optional[Sequence[int]] = None):
    h = ctypes.c_void_p()
    st = _i64(strides) if strides is not None else None
    _check(_lib.load().tensor_partition(ctypes.c_void_p(dev_ptr), DTYPE[dtype], len(bound), _i64(bound), st, _i32(d), ctypes.byref(h)))
    return h


def tensor_relation_block(rel, key: Sequence[int]):
    r = len(key)
    off = ctypes.c_int64()
    b, s = (ctypes.c_int64 * max(1, r))(), (ctypes.c_int64 * max(1, r))()
    _check(_lib.load().tensor_relation_block(rel, _i32(key), ctypes.byref(off), b, s))
    return off.value, list(b[:r]), list(s[:r])


def tensor_relation_destroy(rel) -> None:
    _lib.load().tensor_relation_destroy(rel)


def tr_workspace_bytes(g) -> int:
    n = ctypes.c_size_t()
    _check(_lib.load().tr_workspace_bytes(g, ctypes.byref(n)))
    return n.value


def tr_execute(g, inputs: List, outputs: List, workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> None:
    ia = (ctypes.c_void_p * max(1, len(inputs)))(*[r.value if hasattr(r, "value") else r for r in inputs])
    oa = (ctypes.c_void_p * max(1, len(outputs)))(*[r.value if hasattr(r, "value") else r for r in outputs])
    _check(_lib.load().tr_execute(g, ia, len(inputs), oa, len(outputs), ctypes.c_void_p(workspace_ptr), workspace_bytes,
                                  ctypes.c_void_p(stream)))


def tr_execute_static(g, inputs: List, outputs: List, stream: int = 0) -> None:
    ia = (ctypes.c_void_p * max(1, len(inputs)))(*[r.value if hasattr(r, "value") else r for r in inputs])
    oa = (ctypes.c_void_p * max(1, len(outputs)))(*[r.value if hasattr(r, "value") else r for r in outputs])
    _check(_lib.load().tr_execute_static(g, ia, len(inputs), oa, len(outputs), ctypes.c_void_p(stream)))


def tr_static_workspace_bytes() -> int:
    return int(_lib.load().tr_static_workspace_bytes())


def tr_aggregate(oplus: str, partials_ptr: int, n_agg: int, slab_elems: int, out_rel, stream: int = 0) -> None:
    _check(_lib.load().tr_aggregate(OPLUS[oplus], ctypes.c_void_p(partials_ptr), n_agg, slab_elems, out_rel, ctypes.c_void_p(stream)))


def tr_set_fusion(g, enable: bool) -> None:
    _check(_lib.load().tr_set_fusion(g, 1 if enable else 0))


def tr_set_tiled_partials(g, enable: bool) -> None:
    _check(_lib.load().tr_set_tiled_partials(g, 1 if enable else 0))


def tr_set_fused_attention(g, enable: bool) -> None:
    _check(_lib.load().tr_set_fused_attention(g, 1 if enable else 0))


def tr_set_fused_aggregation(g, enable: bool) -> None:
    _check(_lib.load().tr_set_fused_aggregation(g, 1 if enable else 0))


CONTRACT_KERNELS = {"auto": 0, "staged": 1, "dma": 2}


def tr_set_contract_variant(g, kernel: str = "auto", tile=0, waves: int = 0) -> None:
    """tile: 0 (the library chooses), an int t for t x t, or a pair (tile_m, tile_n)."""
    tm, tn = (tile, tile) if isinstance(tile, int) else tile
    _check(_lib.load().tr_set_contract_variant(g, CONTRACT_KERNELS[kernel], int(tm), int(tn), int(waves)))


# ---- EinDecomp: cost model and choice of the partitioning vectors (host only) -----------------------------
def eg_cost_join(g, vertex: int, d: Sequence[int]) -> int:
    c = ctypes.c_int64()
    _check(_lib.load().eg_cost_join(g, vertex, _i32(d), len(d), ctypes.byref(c)))
    return c.value


def eg_cost_agg(g, vertex: int, d: Sequence[int]) -> int:
    c = ctypes.c_int64()
    _check(_lib.load().eg_cost_agg(g, vertex, _i32(d), len(d), ctypes.byref(c)))
    return c.value


def eg_cost_repart(bound: Sequence[int], d_consumer: Sequence[int], d_producer: Sequence[int]) -> int:
    if not (len(bound) == len(d_consumer) == len(d_producer)):
        raise ValueError("bound and the two cuts must have the same length")
    c = ctypes.c_int64()
    _check(_lib.load().eg_cost_repart(len(bound), _i64(bound), _i32(d_consumer), _i32(d_producer), ctypes.byref(c)))
    return c.value


def eindecomp_viable(g, vertex: int, p: int) -> List[List[int]]:
    lib = _lib.load()
    n = ctypes.c_int()
    _check(lib.eindecomp_viable(g, vertex, p, None, 0, ctypes.byref(n)))
    nl = len(einsum_graph_plan(g, vertex)["labels"])
    buf = (ctypes.c_int32 * max(1, n.value * nl))()
    _check(lib.eindecomp_viable(g, vertex, p, buf, n.value, ctypes.byref(n)))
    return [list(buf[i * nl:(i + 1) * nl]) for i in range(n.value)]


def eindecomp_plan(g, p: int) -> Tuple[int, bool]:
    """Labels every einsum vertex; returns (total cost, whether the labelling is the proven optimum)."""
    c, ex = ctypes.c_int64(), ctypes.c_int()
    _check(_lib.load().eindecomp_plan(g, p, ctypes.byref(c), ctypes.byref(ex)))
    return c.value, bool(ex.value)


def eindecomp_labelling_cost(g) -> dict:
    j, a, r = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(_lib.load().eindecomp_labelling_cost(g, ctypes.byref(j), ctypes.byref(a), ctypes.byref(r)))
    return dict(join=j.value, agg=a.value, repart=r.value, total=j.value + a.value + r.value)


def tr_profile_enable(g, max_launches: int) -> None:
    _check(_lib.load().tr_profile_enable(g, int(max_launches)))


def tr_profile_reset(g) -> None:
    _check(_lib.load().tr_profile_reset(g))


def tr_profile_read(g) -> List[dict]:
    lib = _lib.load()
    n = _check(lib.tr_profile_count(g))
    out = []
    for i in range(n):
        v, s, k, ms = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_float()
        _check(lib.tr_profile_get(g, i, ctypes.byref(v), ctypes.byref(s), ctypes.byref(k), ctypes.byref(ms)))
        slabs = ctypes.c_int64()
        _check(lib.tr_profile_get_slabs(g, i, ctypes.byref(slabs)))
        out.append(dict(vertex=v.value, stage="join" if s.value == 0 else "aggregate", kernel=KERNEL_NAMES[k.value], ms=ms.value,
                        slabs=slabs.value))
    return out


def eg_ceiling_mfma_bf16(sink_ptr: int, cus: int, waves_per_simd: int, iters: int, stream: int = 0) -> float:
    """Enqueues the register-resident MFMA loop; returns its operation count (the caller times it)."""
    fl = ctypes.c_double()
    _check(_lib.load().eg_ceiling_mfma_bf16(ctypes.c_void_p(sink_ptr), cus, waves_per_simd, iters, ctypes.byref(fl), ctypes.c_void_p(stream)))
    return fl.value


def eg_ceiling_mfma_bf16_random(sink_ptr: int, cus: int, iters: int, stream: int = 0) -> float:
    """Enqueues the MFMA loop on pseudo-random operands; returns its operation count (the caller times it)."""
    fl = ctypes.c_double()
    _check(_lib.load().eg_ceiling_mfma_bf16_random(ctypes.c_void_p(sink_ptr), cus, iters, ctypes.byref(fl), ctypes.c_void_p(stream)))
    return fl.value


def eg_ceiling_valu_f32(sink_ptr: int, cus: int, waves_per_simd: int, iters: int, stream: int = 0) -> float:
    """Enqueues the register-resident subtract + fused-multiply-add loop; returns its pair count."""
    n = ctypes.c_double()
    _check(_lib.load().eg_ceiling_valu_f32(ctypes.c_void_p(sink_ptr), cus, waves_per_simd, iters, ctypes.byref(n), ctypes.c_void_p(stream)))
    return n.value


def eg_ceiling_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(_lib.load().eg_ceiling_copy(ctypes.c_void_p(dst_ptr), ctypes.c_void_p(src_ptr), nbytes, ctypes.c_void_p(stream)))


def eg_ceiling_read(dst_ptr: int, src_ptr: int, streams: int, nbytes: int, stream: int = 0) -> None:
    _check(_lib.load().eg_ceiling_read(ctypes.c_void_p(dst_ptr), ctypes.c_void_p(src_ptr), streams, nbytes, ctypes.c_void_p(stream)))
