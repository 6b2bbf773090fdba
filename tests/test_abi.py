"""The C-ABI library loads without a GPU and exports every symbol the header
declares; argument checks that return before any device work are exercised."""
import ctypes
import os
import re

import paper_2104_06700_amd as gnn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "gnnagg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"GNN_API\s+[\w\s\*]+?\b(gnn_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = gnn.load_library()
    declared = _declared_symbols()
    assert len(declared) >= 15
    assert sorted(gnn.EXPORTED_SYMBOLS) == declared
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings_and_defaults():
    names = {gnn.status_string(s) for s in range(7)}
    assert len(names) == 7 and "ok" in names and "unknown status" not in names
    assert gnn.status_string(99) == "unknown status"
    p = gnn.gnn_plan_default_params()
    thr = list(p.thresholds)[:p.n_thresholds]
    assert 0 < p.n_thresholds <= gnn.GNN_MAX_THRESHOLDS
    assert thr == sorted(set(thr)) and thr[0] > 0 and p.hub_chunk > 0


def test_struct_layout_matches_header():
    # gnn_opts: 2 x int32, 2 x int64, 3 pointers, int64, 2 x int32; gnn_plan_params: int32 (+pad), 15 x int64, int64
    assert ctypes.sizeof(gnn.GnnOpts) == 8 + 16 + 24 + 8 + 8
    assert ctypes.sizeof(gnn.GnnPlanParams) == 8 + 15 * 8 + 8
    # gnn_ap_opts: 2 x int32, 3 x int64, 3 pointers, 2 x int32
    assert ctypes.sizeof(gnn.GnnApOpts) == 8 + 24 + 24 + 8
    # gnn_layer_opts: 4 x int32, 3 pointers, int64
    assert ctypes.sizeof(gnn.GnnLayerOpts) == 16 + 24 + 8


def test_argument_checks_that_need_no_device():
    lib = gnn.load_library()
    o = gnn.GnnOpts()
    one = ctypes.c_void_p(16)  # never dereferenced: every call below must return before touching memory
    assert lib.gnn_aggregate_fwd(one, one, None, one, one, -1, 4, 0, ctypes.byref(o)) == gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_aggregate_fwd(one, one, None, one, one, 4, 4, 9, ctypes.byref(o)) == gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_aggregate_fwd(one, one, None, one, one, 0, 4, 0, None) == gnn.GNN_OK
    assert lib.gnn_aggregate_bwd(one, one, None, one, one, 4, 0, 1, None) == gnn.GNN_OK
    assert lib.gnn_aggregate_fwd(None, one, None, one, one, 4, 4, 0, None) == gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_aggregate_fwd_noalloc(one, one, None, one, one, 4, 4, 9, None) == gnn.GNN_ERR_INVALID_ARG
    o.dtype = 5
    assert lib.gnn_aggregate_fwd(one, one, None, one, one, 4, 4, 0, ctypes.byref(o)) == gnn.GNN_ERR_INVALID_ARG
    o.dtype = 0
    o.ldx = 2
    assert lib.gnn_aggregate_fwd(one, one, None, one, one, 4, 4, 0, ctypes.byref(o)) == gnn.GNN_ERR_INVALID_ARG
    o.ldx = 0
    for bad_slices in (3, 5, 16, -1):  # the number of XCD column slices is 1, 2, 4 or 8 (0 = automatic)
        o.max_slices = bad_slices
        assert lib.gnn_aggregate_fwd(one, one, None, one, one, 4, 4, 0, ctypes.byref(o)) == gnn.GNN_ERR_INVALID_ARG
    o.max_slices = 0
    assert lib.gnn_aggregate_bwd(one, one, None, one, one, 4, 4, 1, ctypes.byref(o)) == gnn.GNN_ERR_UNSUPPORTED
    assert lib.gnn_aggregate_bwd(one, one, None, one, one, 4, 4, 3, ctypes.byref(o)) == gnn.GNN_ERR_UNSUPPORTED
    assert lib.gnn_plan_create(None, None, 5, 0, None, None, ctypes.byref(ctypes.c_void_p())) == gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_csr_from_sorted_coo(None, 5, 5, one, 0, None) == gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_calib_copy(one, one, 7, None) == gnn.GNN_ERR_INVALID_ARG
    assert gnn.load_library().gnn_plan_workspace_bytes(None, 4) == 0
    # general primitive
    a = gnn.GnnApOpts()
    bad, ok = gnn.GNN_ERR_INVALID_ARG, gnn.GNN_OK
    assert lib.gnn_ap_fwd(one, one, one, one, one, None, 4, 4, 9, 0, ctypes.byref(a)) == bad       # unknown binop
    assert lib.gnn_ap_fwd(one, one, one, one, one, None, 4, 4, 0, 7, ctypes.byref(a)) == bad       # unknown reduce
    assert lib.gnn_ap_fwd(one, one, one, one, one, one, 4, 4, 0, 0, ctypes.byref(a)) == bad        # winners asked of a sum
    assert lib.gnn_ap_fwd(one, one, one, one, one, None, 0, 4, 0, 0, None) == ok
    assert lib.gnn_ap_fwd(one, one, None, one, one, None, 4, 4, 0, 0, None) == bad                 # add needs f_V
    assert lib.gnn_ap_fwd(one, one, one, None, one, None, 4, 4, 2, 1, None) == bad                 # mul needs f_E
    a.edge_width = 3
    assert lib.gnn_ap_fwd(one, one, one, one, one, None, 4, 4, 0, 0, ctypes.byref(a)) == bad       # width neither d nor 1
    a.edge_width = 0
    a.ldo = 2
    assert lib.gnn_ap_fwd(one, one, one, one, one, None, 4, 4, 0, 0, ctypes.byref(a)) == bad       # stride below d
    a.ldo = 0
    assert lib.gnn_ap_bwd_edge(one, one, None, one, one, one, one, 4, 4, gnn.GNN_BIN_COPY_LHS, ctypes.byref(a)) == bad
    assert lib.gnn_ap_bwd_edge(one, one, None, None, one, one, one, 4, 4, gnn.GNN_BIN_MUL, ctypes.byref(a)) == bad
    assert lib.gnn_ap_bwd_vertex(one, one, one, one, None, 4, 4, 0, ctypes.byref(a)) == bad
    assert lib.gnn_ap_bwd_vertex(one, one, one, one, one, 4, 0, 0, ctypes.byref(a)) == ok
    assert lib.gnn_ap_bwd_vertex_arg(one, one, one, one, one, -1, 4, 4, 0, ctypes.byref(a)) == bad
    # dense update and layer
    assert lib.gnn_matmul(one, 4, 0, one, 4, 0, one, 2, 4, 4, 4, None, 0, None, 0, None) == bad      # ldc < N
    assert lib.gnn_matmul(None, 4, 0, one, 4, 0, one, 4, 4, 4, 4, None, 0, None, 0, None) == bad
    assert lib.gnn_matmul(one, 4, 0, one, 4, 0, one, 4, 0, 4, 4, None, 0, None, 0, None) == ok
    assert lib.gnn_matmul_workspace_bytes(100, 47, 2_000_000) > 0 and lib.gnn_matmul_workspace_bytes(2_000_000, 256, 100) == 0
    lo = gnn.GnnLayerOpts()
    assert lib.gnn_sage_layer_fwd(one, one, one, one, None, one, one, 4, 4, 4, None) == bad
    assert lib.gnn_sage_layer_fwd(one, one, one, one, None, one, one, 4, 4, 4, ctypes.byref(lo)) == gnn.GNN_ERR_UNSUPPORTED
    lo.order = 5
    assert lib.gnn_sage_layer_bwd(one, one, one, one, one, one, one, one, one, one, 4, 4, 4, ctypes.byref(lo)) == bad
    assert lib.gnn_sage_layer_saved_elems(10, 3, 5, 0) == 30 and lib.gnn_sage_layer_saved_elems(10, 5, 3, 0) == 40  # rows padded to 4 floats
    assert lib.gnn_sage_layer_saved_elems(10, 5, 3, 1) == 50
    assert lib.gnn_sage_layer_workspace_bytes(1000, 8, 4, 1, 0) >= 1000 * 4 * 4 * 2


def test_packed_copy_sizes_and_argument_checks_that_need_no_device():
    """gnn_packed_bytes is host arithmetic: one table of whole 128-byte lines per line of a row (two to 256
    lines; the last one padded)."""
    assert gnn.gnn_packed_bytes(1000, 100, gnn.GNN_F32) == 1000 * 4 * 128
    assert gnn.gnn_packed_bytes(1000, 256, gnn.GNN_F32) == 1000 * 256 * 4
    assert gnn.gnn_packed_bytes(1000, 50, gnn.GNN_F32) == 1000 * 64 * 4
    assert gnn.gnn_packed_bytes(1000, 47, gnn.GNN_F32) == 1000 * 2 * 128
    assert gnn.gnn_packed_bytes(7, 65, gnn.GNN_BF16) == 7 * 2 * 128
    assert gnn.gnn_packed_bytes(1000, 32, gnn.GNN_F32) == 0 and gnn.gnn_packed_bytes(1000, 64, gnn.GNN_BF16) == 0
    assert gnn.gnn_packed_bytes(1000, 256 * 32, gnn.GNN_F32) == 1000 * 256 * 32 * 4
    assert gnn.gnn_packed_bytes(1000, 256 * 32 + 1, gnn.GNN_F32) == 0
    assert gnn.gnn_packed_bytes(0, 100, gnn.GNN_F32) == 0 and gnn.gnn_packed_bytes(-3, 100, gnn.GNN_F32) == 0
    assert gnn.gnn_packed_bytes(10, 100, 7) == 0
    lib = gnn.load_library()
    one = ctypes.c_void_p(128)  # never dereferenced
    o = gnn.GnnOpts()
    # the row order of a packed copy is a plan's: without one the calls refuse before any device work
    assert lib.gnn_pack_rows(one, one, one, one, 1 << 20, 100, 100, 0, 0, ctypes.byref(o)) == gnn.GNN_ERR_UNSUPPORTED
    assert lib.gnn_aggregate_packed(one, one, None, one, 1 << 20, one, 100, 100, 0, 0, ctypes.byref(o)) == gnn.GNN_ERR_UNSUPPORTED
    assert lib.gnn_pack_rows(one, one, one, one, 1 << 20, -1, 100, 0, 0, None) == gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_pack_rows(one, one, one, one, 1 << 20, 100, 100, 9, 0, None) == gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_aggregate_packed(one, one, None, None, 0, one, 0, 100, 0, 0, None) == gnn.GNN_OK
    assert lib.gnn_aggregate_packed(one, one, None, None, 0, one, 5, 100, 0, 0, None) == gnn.GNN_ERR_INVALID_ARG


def test_calibration_calls_check_their_arguments_without_a_device():
    lib = gnn.load_library()
    one = ctypes.c_void_p(128)  # never dereferenced
    bad = gnn.GNN_ERR_INVALID_ARG
    assert lib.gnn_calib_gather(None, 10, one, 1 << 28, one, 1 << 23, None) == bad
    assert lib.gnn_calib_gather(one, 0, one, 1 << 28, one, 1 << 23, None) == bad           # empty table
    assert lib.gnn_calib_gather(one, 10, one, 1 << 20, one, 1 << 23, None) == bad           # fewer than 16 lines per lane group
    assert lib.gnn_calib_gather(one, 10, one, 1 << 28, one, (1 << 23) - 1, None) == bad     # output too small
    assert lib.gnn_calib_gather(ctypes.c_void_p(64), 10, one, 1 << 28, one, 1 << 23, None) == bad  # table not line-aligned
    assert lib.gnn_plan_bind_edge_weights(None, one, None) == bad                           # no plan
