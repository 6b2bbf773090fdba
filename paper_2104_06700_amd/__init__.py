"""MI355X-native neighbour aggregation (forward over CSR, backward over the
transposed graph; sum-type variants on the hot path, the whole operator table
through the gnn_ap_* calls) behind the C ABI declared in include/gnnagg.h.

The Python layer only marshals arguments; all arithmetic and all graph
preprocessing (row pointers, transpose, degree binning) run in the library's
HIP kernels.
"""
from .binding import (  # noqa: F401
    GNN_OK, GNN_ERR_INVALID_ARG, GNN_ERR_UNSUPPORTED, GNN_ERR_ALLOC, GNN_ERR_LAUNCH, GNN_ERR_INVALID_GRAPH,
    GNN_ERR_SCRATCH_CAPACITY, GNN_NOALLOC_SCRATCH_BYTES, gnn_aggregate_fwd_noalloc, gnn_packed_bytes, gnn_pack_rows, gnn_aggregate_packed,
    GNN_SUM, GNN_MEAN, GNN_GCN_SYM, GNN_SAGE_GCN, GNN_F32, GNN_BF16, GNN_MAX_THRESHOLDS, GNN_FLAG_NO_COLUMN_SLICES, GNN_FLAG_NO_PADDED_COPY, GNN_FLAG_FORCE_PADDED_COPY, GNN_FLAG_PADDED_ROWS, GNN_FLAG_NO_COLD_HINTS, GNN_FLAG_FORCE_COLD_HINTS, GNN_FLAG_NO_RANK_ORDER, GNN_FLAG_NO_SLICE_TABLES, GNN_FLAG_NO_SOURCE_BLOCKS, GNN_FLAG_NO_SHORT_ROW_OVERLAP, GNN_FLAG_NO_DENSE_TAIL, GNN_LAYER_FORCE_PRODUCER_LAYOUT, GNN_LAYER_NO_PRODUCER_LAYOUT, GNN_LAYER_NO_GATE_FOLD, GnnBlockingParams, EXPORTED_SYMBOLS, LIB_PATH,
    GNN_BIN_ADD, GNN_BIN_SUB, GNN_BIN_MUL, GNN_BIN_DIV, GNN_BIN_COPY_LHS, GNN_BIN_COPY_RHS, GNN_RED_SUM, GNN_RED_MAX, GNN_RED_MIN,
    GnnError, GnnOpts, GnnApOpts, GnnLayerOpts, GnnPlanParams, Plan,
    load_library, status_string, make_plan_params,
    gnn_aggregate_fwd, gnn_aggregate_bwd, gnn_csr_from_sorted_coo, gnn_transpose_csr, gnn_validate_csr,
    gnn_plan_default_params, gnn_plan_create, gnn_calib_copy, gnn_calib_gather,
    gnn_ap_fwd, gnn_ap_bwd_vertex, gnn_ap_bwd_vertex_arg, gnn_ap_bwd_edge, gnn_matmul, gnn_matmul_workspace_bytes,
    gnn_sage_layer_fwd, gnn_sage_layer_bwd, gnn_sage_layer_saved_elems, gnn_sage_layer_workspace_bytes,
)
from .graph import DeviceGraph, build_device_graph  # noqa: F401
