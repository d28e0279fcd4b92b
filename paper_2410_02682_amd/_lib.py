"""Loads libeindecomp.so and declares the C ABI of include/eindecomp.h for ctypes.

There is no fallback: if the library has not been built, importing the binding raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("EINDECOMP_LIB") or os.path.join(HERE, "libeindecomp.so")   # override: an alternate build of the same ABI

EG_MAX_RANK = 8
EG_MAX_LABELS = 12

c_i32p = ctypes.POINTER(ctypes.c_int32)
c_i64p = ctypes.POINTER(ctypes.c_int64)


class PlanView(ctypes.Structure):
    _fields_ = [
        ("n_labels", ctypes.c_int32),
        ("labels", ctypes.c_char * EG_MAX_LABELS),
        ("bound", ctypes.c_int64 * EG_MAX_LABELS),
        ("d", ctypes.c_int32 * EG_MAX_LABELS),
        ("rank_x", ctypes.c_int32), ("rank_y", ctypes.c_int32), ("rank_z", ctypes.c_int32),
        ("d_x", ctypes.c_int32 * EG_MAX_RANK), ("d_y", ctypes.c_int32 * EG_MAX_RANK), ("d_z", ctypes.c_int32 * EG_MAX_RANK),
        ("bound_z", ctypes.c_int64 * EG_MAX_RANK),
        ("block_x", ctypes.c_int64 * EG_MAX_RANK), ("block_y", ctypes.c_int64 * EG_MAX_RANK), ("block_z", ctypes.c_int64 * EG_MAX_RANK),
        ("n_tuples", ctypes.c_int64), ("n_agg", ctypes.c_int64), ("n_groups", ctypes.c_int64),
        ("kernel", ctypes.c_int32), ("repart_x", ctypes.c_int32), ("repart_y", ctypes.c_int32),
        ("key", c_i32p), ("key_x", c_i32p), ("key_y", c_i32p), ("key_z", c_i32p),
        ("agg_idx", c_i32p), ("group", c_i32p),
        ("off_x", c_i64p), ("off_y", c_i64p), ("off_z", c_i64p),
    ]


EXPORTS = {
    # name: (restype, argtypes)
    "einsum_graph_create": (ctypes.c_int, [ctypes.POINTER(ctypes.c_void_p)]),
    "einsum_graph_add_input": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, c_i64p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]),
    "einsum_graph_add_einsum": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_char_p, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                               ctypes.POINTER(ctypes.c_int), ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]),
    "einsum_graph_set_partition": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, c_i32p, ctypes.c_int]),
    "einsum_graph_mark_output": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "einsum_graph_plan": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(PlanView)]),
    "einsum_graph_num_vertices": (ctypes.c_int, [ctypes.c_void_p]),
    "einsum_graph_destroy": (None, [ctypes.c_void_p]),
    "tensor_partition": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, c_i64p, c_i64p, c_i32p, ctypes.POINTER(ctypes.c_void_p)]),
    "tensor_relation_block": (ctypes.c_int, [ctypes.c_void_p, c_i32p, c_i64p, c_i64p, c_i64p]),
    "tensor_relation_destroy": (None, [ctypes.c_void_p]),
    "tr_workspace_bytes": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t)]),
    "tr_execute": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                  ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "tr_execute_static": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                         ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p]),
    "tr_static_workspace_bytes": (ctypes.c_size_t, []),
    "tr_aggregate": (ctypes.c_int, [ctypes.c_int, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]),
    "tr_set_fusion": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "tr_set_fused_attention": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "tr_set_tiled_partials": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "tr_set_fused_aggregation": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "tr_set_contract_variant": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]),
    "tr_profile_enable": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "tr_profile_reset": (ctypes.c_int, [ctypes.c_void_p]),
    "tr_profile_count": (ctypes.c_int, [ctypes.c_void_p]),
    "tr_profile_get": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int),
                                      ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)]),
    "tr_profile_get_slabs": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]),
    "eg_cost_join": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, c_i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]),
    "eg_cost_agg": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, c_i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]),
    "eg_cost_repart": (ctypes.c_int, [ctypes.c_int, c_i64p, c_i32p, c_i32p, ctypes.POINTER(ctypes.c_int64)]),
    "eindecomp_viable": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, c_i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]),
    "eindecomp_plan": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int)]),
    "eindecomp_labelling_cost": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
    "eg_ceiling_mfma_bf16": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]),
    "eg_ceiling_mfma_bf16_random": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]),
    "eg_ceiling_valu_f32": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]),
    "eg_ceiling_copy": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]),
    "eg_ceiling_read": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_void_p]),
    "eg_last_error": (ctypes.c_char_p, []),
}

_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2410_02682_amd.build, or "
                "__graft_entry__.build()).  There is no CPU fallback.")
        # torch ships its own HIP runtime; it must be the one already resident when this library's
        # libamdhip64 dependency is resolved, or the process ends up with two runtimes that do not share
        # device state (streams, allocations, code objects).
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib
