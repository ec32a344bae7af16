"""gnnhot: one GPU's share of a full-neighbourhood GNN training step under one-hop graph
masking (GraNNDis, arXiv 2311.06837) as hand-written HIP kernels for MI355X behind a C ABI.

``binding`` mirrors include/gnnhot.h with torch tensors; ``model`` sequences the calls for one
partition; ``build`` compiles the library.  There is no CPU fallback.
"""
from .binding import (GNN_BF16, GNN_F32, GNN_NORM_MEAN, GNN_NORM_SYM, GnnError, Graph, Workspace, gnn_build_active_sets,
                      gnn_linear_bwd, gnn_linear_fwd, gnn_make_bitmap, gnn_masked_spmm_bwd, gnn_masked_spmm_fwd, gnn_masked_spmm_fwd_add,
                      gnn_norm_scales, gnn_sample_boundary, gnn_softmax_ce, gnn_version, gnn_extract_partition, gnn_gather_rows, gnn_expand_row_ptr,
                      gnn_extract_sampled_partition, gnn_eas_traverse, gnn_layer_edge_mask, gnn_transpose_edge_mask,
                      gnn_layer_edge_mask_transposed, gnn_layer_norm_relu_fwd, gnn_layer_norm_relu_bwd, gnn_add_rows, gnn_add_rows_masked, gnn_bias_grad, gnn_linear_bwd_input,
                      gnn_linear_fwd_static, gnn_linear_bwd_input2, gnn_die_mapping, gnn_fused_layer_fwd)
from .model import MaskedGNN, ResSAGEPlus, row_stride

__all__ = ["GNN_BF16", "GNN_F32", "GNN_NORM_MEAN", "GNN_NORM_SYM", "GnnError", "Graph", "Workspace", "MaskedGNN", "row_stride",
           "gnn_build_active_sets", "gnn_linear_bwd", "gnn_linear_fwd", "gnn_make_bitmap", "gnn_masked_spmm_bwd",
           "gnn_masked_spmm_fwd", "gnn_masked_spmm_fwd_add", "gnn_norm_scales", "gnn_sample_boundary", "gnn_softmax_ce", "gnn_version",
           "gnn_extract_partition", "gnn_gather_rows", "gnn_expand_row_ptr", "gnn_extract_sampled_partition", "gnn_eas_traverse",
           "gnn_layer_edge_mask", "gnn_transpose_edge_mask", "gnn_layer_edge_mask_transposed",
           "gnn_layer_norm_relu_fwd", "gnn_layer_norm_relu_bwd", "gnn_add_rows", "gnn_add_rows_masked", "gnn_bias_grad", "gnn_linear_bwd_input", "ResSAGEPlus",
           "gnn_linear_fwd_static", "gnn_linear_bwd_input2", "gnn_die_mapping", "gnn_fused_layer_fwd"]
