"""MI355X tensor-relational einsum executor: Python binding over libeindecomp.so (C ABI in include/eindecomp.h)."""
from .api import (EgError, einsum_graph_create, einsum_graph_add_input, einsum_graph_add_einsum,
                  einsum_graph_set_partition, einsum_graph_mark_output, einsum_graph_plan, einsum_graph_destroy,
                  tensor_partition, tensor_relation_block, tensor_relation_destroy,
                  tr_workspace_bytes, tr_execute, tr_execute_static, tr_static_workspace_bytes, tr_aggregate, tr_set_fusion, tr_set_fused_aggregation, tr_set_fused_attention, tr_set_tiled_partials, tr_set_contract_variant, tr_profile_enable, tr_profile_reset, tr_profile_read,
                  eg_cost_join, eg_cost_agg, eg_cost_repart, eindecomp_viable, eindecomp_plan, eindecomp_labelling_cost,
                  eg_ceiling_mfma_bf16, eg_ceiling_mfma_bf16_random, eg_ceiling_valu_f32, eg_ceiling_copy, eg_ceiling_read)
