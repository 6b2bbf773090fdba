"""ctypes binding of libgnnagg.so: same names as the C ABI, argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used here
for device memory and the current stream.  There is no CPU fallback: if the
shared library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgnnagg.so")

GNN_OK, GNN_ERR_INVALID_ARG, GNN_ERR_UNSUPPORTED, GNN_ERR_ALLOC, GNN_ERR_LAUNCH, GNN_ERR_INVALID_GRAPH = range(6)
GNN_ERR_SCRATCH_CAPACITY = 6
GNN_NOALLOC_SCRATCH_BYTES = 32 << 20
GNN_SUM, GNN_MEAN, GNN_GCN_SYM, GNN_SAGE_GCN = 0, 1, 2, 3
GNN_F32, GNN_BF16 = 0, 1
GNN_MAX_THRESHOLDS = 15
GNN_FLAG_NO_COLUMN_SLICES = 1
GNN_FLAG_NO_PADDED_COPY = 2
GNN_FLAG_FORCE_PADDED_COPY = 4
GNN_FLAG_PADDED_ROWS = 8
GNN_FLAG_NO_COLD_HINTS = 16
GNN_FLAG_FORCE_COLD_HINTS = 32
GNN_FLAG_NO_RANK_ORDER = 64
GNN_FLAG_NO_SLICE_TABLES = 128
GNN_FLAG_NO_SOURCE_BLOCKS = 256
GNN_FLAG_NO_SHORT_ROW_OVERLAP = 512
GNN_FLAG_NO_DENSE_TAIL = 1024
GNN_BIN_ADD, GNN_BIN_SUB, GNN_BIN_MUL, GNN_BIN_DIV, GNN_BIN_COPY_LHS, GNN_BIN_COPY_RHS = range(6)
GNN_RED_SUM, GNN_RED_MAX, GNN_RED_MIN = range(3)

EXPORTED_SYMBOLS = (
    "gnn_aggregate_fwd", "gnn_aggregate_bwd", "gnn_aggregate_fwd_noalloc", "gnn_packed_bytes", "gnn_pack_rows",
    "gnn_aggregate_packed", "gnn_csr_from_sorted_coo", "gnn_transpose_csr",
    "gnn_validate_csr", "gnn_plan_default_params", "gnn_plan_create", "gnn_plan_destroy",
    "gnn_plan_sizes", "gnn_plan_export", "gnn_plan_gather_share", "gnn_plan_workspace_bytes", "gnn_plan_reserve",
    "gnn_plan_prepare", "gnn_plan_set_blocking", "gnn_plan_bind_edge_weights", "gnn_plan_blocked_sizes", "gnn_plan_export_blocked",
    "gnn_ap_fwd", "gnn_ap_bwd_vertex", "gnn_ap_bwd_vertex_arg", "gnn_ap_bwd_edge",
    "gnn_matmul", "gnn_matmul_workspace_bytes",
    "gnn_sage_layer_fwd", "gnn_sage_layer_bwd", "gnn_sage_layer_saved_elems", "gnn_sage_layer_workspace_bytes",
    "gnn_status_string", "gnn_calib_copy", "gnn_calib_gather",
)


class GnnOpts(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32), ("indptr_is_64", ctypes.c_int32),
        ("ldx", ctypes.c_int64), ("ldy", ctypes.c_int64),
        ("stream", ctypes.c_void_p), ("plan", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_int64),
        ("flags", ctypes.c_int32), ("max_slices", ctypes.c_int32),
    ]


class GnnApOpts(ctypes.Structure):
    _fields_ = [
        ("indptr_is_64", ctypes.c_int32), ("edge_width", ctypes.c_int32),
        ("ldv", ctypes.c_int64), ("lde", ctypes.c_int64), ("ldo", ctypes.c_int64),
        ("edge_ids", ctypes.c_void_p), ("stream", ctypes.c_void_p), ("plan", ctypes.c_void_p),
        ("flags", ctypes.c_int32), ("max_slices", ctypes.c_int32),
    ]


class GnnLayerOpts(ctypes.Structure):
    _fields_ = [
        ("indptr_is_64", ctypes.c_int32), ("relu", ctypes.c_int32), ("order", ctypes.c_int32), ("flags", ctypes.c_int32),
        ("stream", ctypes.c_void_p), ("plan", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_int64),
    ]


class GnnPlanParams(ctypes.Structure):
    _fields_ = [
        ("n_thresholds", ctypes.c_int32),
        ("thresholds", ctypes.c_int64 * GNN_MAX_THRESHOLDS),
        ("hub_chunk", ctypes.c_int64),
    ]


class GnnBlockingParams(ctypes.Structure):
    _fields_ = [("min_degree", ctypes.c_int64), ("hot_lines", ctypes.c_int64), ("block_lines", ctypes.c_int64),
                ("max_piece", ctypes.c_int64), ("rest_min_count", ctypes.c_int64)]


class GnnError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed: {status_string(status)} (status {status})")


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.gnn_aggregate_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, ctypes.POINTER(GnnOpts)]
        lib.gnn_aggregate_bwd.argtypes = lib.gnn_aggregate_fwd.argtypes
        lib.gnn_aggregate_fwd_noalloc.argtypes = lib.gnn_aggregate_fwd.argtypes
        lib.gnn_packed_bytes.argtypes = [i64, i64, i32]
        lib.gnn_packed_bytes.restype = i64
        lib.gnn_pack_rows.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, ctypes.POINTER(GnnOpts)]
        lib.gnn_aggregate_packed.argtypes = [vp, vp, vp, vp, i64, vp, i64, i64, i32, i32, ctypes.POINTER(GnnOpts)]
        lib.gnn_csr_from_sorted_coo.argtypes = [vp, i64, i64, vp, i32, vp]
        lib.gnn_transpose_csr.argtypes = [vp, vp, vp, i64, i32, vp, vp, vp, vp, vp]
        lib.gnn_validate_csr.argtypes = [vp, vp, i64, i64, i32, vp]
        lib.gnn_plan_default_params.argtypes = [ctypes.POINTER(GnnPlanParams)]
        lib.gnn_plan_default_params.restype = None
        lib.gnn_plan_create.argtypes = [vp, vp, i64, i32, ctypes.POINTER(GnnPlanParams), vp, ctypes.POINTER(vp)]
        lib.gnn_plan_destroy.argtypes = [vp]
        lib.gnn_plan_destroy.restype = None
        lib.gnn_plan_sizes.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(i64)]
        lib.gnn_plan_export.argtypes = [vp, vp, vp, vp, vp]
        lib.gnn_plan_gather_share.argtypes = [vp, i64]
        lib.gnn_plan_gather_share.restype = ctypes.c_double
        lib.gnn_plan_workspace_bytes.argtypes = [vp, i64]
        lib.gnn_plan_workspace_bytes.restype = i64
        lib.gnn_plan_reserve.argtypes = [vp, i64]
        lib.gnn_plan_prepare.argtypes = [vp, vp, i32, i32, i64, i32, vp]
        lib.gnn_plan_set_blocking.argtypes = [vp, ctypes.POINTER(GnnBlockingParams)]
        lib.gnn_plan_bind_edge_weights.argtypes = [vp, vp, vp]
        lib.gnn_plan_blocked_sizes.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64),
                                               ctypes.POINTER(ctypes.c_int32)]
        lib.gnn_plan_export_blocked.argtypes = [vp, vp, vp, vp, vp, vp]
        ap = ctypes.POINTER(GnnApOpts)
        lib.gnn_ap_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i32, i32, ap]
        lib.gnn_ap_bwd_vertex.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, ap]
        lib.gnn_ap_bwd_vertex_arg.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, ap]
        lib.gnn_ap_bwd_edge.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i32, ap]
        lib.gnn_matmul.argtypes = [vp, i64, i32, vp, i64, i32, vp, i64, i64, i64, i64, vp, i32, vp, i64, vp]
        lib.gnn_matmul_workspace_bytes.argtypes = [i64, i64, i64]
        lib.gnn_matmul_workspace_bytes.restype = i64
        lp = ctypes.POINTER(GnnLayerOpts)
        lib.gnn_sage_layer_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, lp]
        lib.gnn_sage_layer_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, lp]
        lib.gnn_sage_layer_saved_elems.argtypes = [i64, i64, i64, i32]
        lib.gnn_sage_layer_saved_elems.restype = i64
        lib.gnn_sage_layer_workspace_bytes.argtypes = [i64, i64, i64, i32, i32]
        lib.gnn_sage_layer_workspace_bytes.restype = i64
        lib.gnn_status_string.argtypes = [i32]
        lib.gnn_status_string.restype = ctypes.c_char_p
        lib.gnn_calib_copy.argtypes = [vp, vp, i64, vp]
        lib.gnn_calib_gather.argtypes = [vp, i64, vp, i64, vp, i64, vp]
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().gnn_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous() and t.dim() == 1:
        raise ValueError("1-D arguments must be contiguous")
    return t.data_ptr() if t.numel() > 0 else (t.data_ptr() or None)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _check(fn: str, status: int) -> None:
    if status != GNN_OK:
        raise GnnError(fn, status)


def _call_allocating(fn: str, call) -> None:
    """Library calls that hipMalloc can fail only because torch's caching allocator is
    sitting on freed blocks: hand those back to the driver and try once more."""
    status = call()
    if status == GNN_ERR_ALLOC:
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        status = call()
    _check(fn, status)


def _is64(indptr: torch.Tensor) -> int:
    if indptr.dtype == torch.int64:
        return 1
    if indptr.dtype == torch.int32:
        return 0
    raise TypeError("indptr must be int32 or int64")


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GNN_F32
    if t.dtype == torch.bfloat16:
        return GNN_BF16
    raise TypeError("features must be float32 or bfloat16")


class Plan:
    """Owner of a gnn_plan handle (destroyed with the object)."""

    def __init__(self, handle: int, n_thresholds: int):
        self.handle = handle
        self.n_thresholds = n_thresholds

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.gnn_plan_destroy(h)

    def sizes(self):
        n = ctypes.c_int64(); b = ctypes.c_int32(); c = ctypes.c_int64()
        _check("gnn_plan_sizes", load_library().gnn_plan_sizes(self.handle, ctypes.byref(n), ctypes.byref(b), ctypes.byref(c)))
        return n.value, b.value, c.value

    def export(self):
        """Host copies: (bin_offsets int64[n_bins+1], row_perm int32[N], chunks int64[n_chunks,3], col_counts int32[N])."""
        import numpy as np
        n, b, c = self.sizes()
        bin_offsets = np.zeros(b + 1, dtype=np.int64)
        row_perm = np.zeros(n, dtype=np.int32)
        chunks = np.zeros((c, 3), dtype=np.int64)
        col_counts = np.zeros(n, dtype=np.int32)
        _check("gnn_plan_export", load_library().gnn_plan_export(
            self.handle, bin_offsets.ctypes.data, row_perm.ctypes.data if n else None,
            chunks.ctypes.data if c else None, col_counts.ctypes.data if n else None))
        return bin_offsets, row_perm, chunks, col_counts

    def set_blocking(self, min_degree=0, hot_lines=0, block_lines=0, max_piece=0, rest_min_count=0) -> None:
        """Parameters of the source-blocked layout of the long rows (zeros: automatic; min_degree < 0: off)."""
        p = GnnBlockingParams(int(min_degree), int(hot_lines), int(block_lines), int(max_piece), int(rest_min_count))
        _check("gnn_plan_set_blocking", load_library().gnn_plan_set_blocking(self.handle, ctypes.byref(p)))

    def bind_edge_weights(self, edge_w, stream=None) -> None:
        """Declares `edge_w` (fp32 device tensor in the plan's CSR order, or None) static: calls that pass this
        tensor serve their long rows as source-blocked pieces from a plan-owned copy.  Bind again after the
        contents change."""
        ptr = None
        if edge_w is not None:
            if edge_w.dtype != torch.float32 or not edge_w.is_contiguous() or not edge_w.is_cuda:
                raise ValueError("edge_w: contiguous fp32 device tensor expected")
            ptr = edge_w.data_ptr()
        _check("gnn_plan_bind_edge_weights", load_library().gnn_plan_bind_edge_weights(self.handle, ptr, _stream(stream)))

    def blocked_sizes(self):
        """(rows served as pieces, their edges, pieces, blocks); zeros when the plan has no such layout (yet)."""
        r = ctypes.c_int64(); e = ctypes.c_int64(); p = ctypes.c_int64(); b = ctypes.c_int32()
        _check("gnn_plan_blocked_sizes", load_library().gnn_plan_blocked_sizes(
            self.handle, ctypes.byref(r), ctypes.byref(e), ctypes.byref(p), ctypes.byref(b)))
        return r.value, e.value, p.value, b.value

    def export_blocked(self):
        """Host copies of the source-blocked layout: (indices int32[E_b], epos uint32[E_b], pieces int32[P,4],
        rowbase uint32[R+1], rank int32[N])."""
        import numpy as np
        r, e, p, _ = self.blocked_sizes()
        n = self.sizes()[0]
        indices = np.zeros(e, dtype=np.int32); epos = np.zeros(e, dtype=np.uint32)
        pieces = np.zeros((p, 4), dtype=np.int32); rowbase = np.zeros(r + 1 if p else 0, dtype=np.uint32)
        rank = np.zeros(n, dtype=np.int32)
        _check("gnn_plan_export_blocked", load_library().gnn_plan_export_blocked(
            self.handle, indices.ctypes.data if e else None, epos.ctypes.data if e else None,
            pieces.ctypes.data if p else None, rowbase.ctypes.data if p else None, rank.ctypes.data if n else None))
        return indices, epos, pieces, rowbase, rank

    def gather_share(self, K: int) -> float:
        return float(load_library().gnn_plan_gather_share(self.handle, int(K)))

    def workspace_bytes(self, F: int) -> int:
        return int(load_library().gnn_plan_workspace_bytes(self.handle, int(F)))

    def reserve(self, F: int) -> None:
        _call_allocating("gnn_plan_reserve", lambda: load_library().gnn_plan_reserve(self.handle, int(F)))

    def prepare(self, indices: torch.Tensor, op: int, backward: bool, F: int, dtype=torch.float32, stream=None) -> None:
        code = GNN_BF16 if dtype == torch.bfloat16 else GNN_F32
        _call_allocating("gnn_plan_prepare", lambda: load_library().gnn_plan_prepare(
            self.handle, _ptr(indices), int(op), 1 if backward else 0, int(F), code, _stream(stream)))


def gnn_plan_default_params() -> GnnPlanParams:
    p = GnnPlanParams()
    load_library().gnn_plan_default_params(ctypes.byref(p))
    return p


def make_plan_params(thresholds: Sequence[int], hub_chunk: int) -> GnnPlanParams:
    p = GnnPlanParams()
    p.n_thresholds = len(thresholds)
    for i, t in enumerate(thresholds):
        p.thresholds[i] = int(t)
    p.hub_chunk = int(hub_chunk)
    return p


def gnn_plan_create(indptr: torch.Tensor, indices: torch.Tensor, N: int,
                    params: Optional[GnnPlanParams] = None, stream=None) -> Plan:
    out = ctypes.c_void_p()
    _call_allocating("gnn_plan_create", lambda: load_library().gnn_plan_create(
        _ptr(indptr), _ptr(indices), int(N), _is64(indptr), ctypes.byref(params) if params is not None else None,
        _stream(stream), ctypes.byref(out)))
    k = params.n_thresholds if params is not None else gnn_plan_default_params().n_thresholds
    return Plan(out.value, k)


def _aggregate(fn_name, indptr, indices, edge_w, X, Y, N, F, op, plan, stream, workspace, ldx, ldy, flags=0, max_slices=0):
    lib = load_library()
    if X.dtype != Y.dtype:
        raise TypeError("input and output features must have the same dtype")
    o = GnnOpts()
    o.dtype = _dtype_code(X)
    o.indptr_is_64 = _is64(indptr)
    o.ldx = int(ldx if ldx is not None else (X.stride(0) if X.dim() == 2 and X.shape[0] > 1 else 0))
    o.ldy = int(ldy if ldy is not None else (Y.stride(0) if Y.dim() == 2 and Y.shape[0] > 1 else 0))
    o.stream = _stream(stream)
    o.plan = plan.handle if plan is not None else None
    o.flags = int(flags)
    o.max_slices = int(max_slices)
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    _call_allocating(fn_name, lambda: getattr(lib, fn_name)(_ptr(indptr), _ptr(indices), _ptr(edge_w), _ptr(X), _ptr(Y),
                                                            int(N), int(F), int(op), ctypes.byref(o)))


def gnn_aggregate_fwd(indptr, indices, edge_w, X, Y, N, F, op, plan: Optional[Plan] = None, stream=None,
                      workspace=None, ldx=None, ldy=None, flags=0, max_slices=0) -> None:
    """Y[v] = scale_v * sum_e c_e X[indices[e]] over the CSR by destination (see include/gnnagg.h)."""
    _aggregate("gnn_aggregate_fwd", indptr, indices, edge_w, X, Y, N, F, op, plan, stream, workspace, ldx, ldy, flags,
               max_slices)


def gnn_aggregate_fwd_noalloc(indptr, indices, edge_w, X, Y, N, F, op, plan: Optional[Plan] = None, stream=None,
                              ldx=None, ldy=None, flags=0, max_slices=0) -> None:
    """gnn_aggregate_fwd that allocates nothing: hub partial sums in the library's fixed scratch array."""
    lib = load_library()
    if X.dtype != Y.dtype:
        raise TypeError("input and output features must have the same dtype")
    o = GnnOpts()
    o.dtype = _dtype_code(X)
    o.indptr_is_64 = _is64(indptr)
    o.ldx = int(ldx if ldx is not None else (X.stride(0) if X.dim() == 2 and X.shape[0] > 1 else 0))
    o.ldy = int(ldy if ldy is not None else (Y.stride(0) if Y.dim() == 2 and Y.shape[0] > 1 else 0))
    o.stream = _stream(stream)
    o.plan = plan.handle if plan is not None else None
    o.flags = int(flags)
    o.max_slices = int(max_slices)
    # no retry through torch's allocator here: this call must not allocate, so ALLOC cannot come back
    _check("gnn_aggregate_fwd_noalloc", lib.gnn_aggregate_fwd_noalloc(
        _ptr(indptr), _ptr(indices), _ptr(edge_w), _ptr(X), _ptr(Y), int(N), int(F), int(op), ctypes.byref(o)))


def gnn_packed_bytes(N, F, dtype) -> int:
    """Bytes of a caller-kept packed copy of an [N, F] matrix (0: such rows are not laid out as tables)."""
    return int(load_library().gnn_packed_bytes(int(N), int(F), int(dtype)))


def gnn_pack_rows(indptr, indices, X, packed, N, F, op, backward, plan: Plan, stream=None, ldx=None) -> None:
    """Writes the packed copy of X that gnn_aggregate_packed gathers from (see include/gnnagg.h)."""
    lib = load_library()
    o = GnnOpts()
    o.dtype = _dtype_code(X)
    o.indptr_is_64 = _is64(indptr)
    o.ldx = int(ldx if ldx is not None else (X.stride(0) if X.dim() == 2 and X.shape[0] > 1 else 0))
    o.stream = _stream(stream)
    o.plan = plan.handle if plan is not None else None
    _call_allocating("gnn_pack_rows", lambda: lib.gnn_pack_rows(
        _ptr(indptr), _ptr(indices), _ptr(X), _ptr(packed), packed.numel() * packed.element_size(), int(N), int(F),
        int(op), int(bool(backward)), ctypes.byref(o)))


def gnn_aggregate_packed(indptr, indices, edge_w, packed, Y, N, F, op, backward, plan: Plan, stream=None, workspace=None,
                         ldy=None, flags=0) -> None:
    """gnn_aggregate_fwd / _bwd reading a packed copy in place of the gathered matrix (see include/gnnagg.h)."""
    lib = load_library()
    o = GnnOpts()
    o.dtype = _dtype_code(Y)
    o.indptr_is_64 = _is64(indptr)
    o.ldy = int(ldy if ldy is not None else (Y.stride(0) if Y.dim() == 2 and Y.shape[0] > 1 else 0))
    o.stream = _stream(stream)
    o.plan = plan.handle if plan is not None else None
    o.flags = int(flags)
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    _call_allocating("gnn_aggregate_packed", lambda: lib.gnn_aggregate_packed(
        _ptr(indptr), _ptr(indices), _ptr(edge_w), _ptr(packed), packed.numel() * packed.element_size(), _ptr(Y),
        int(N), int(F), int(op), int(bool(backward)), ctypes.byref(o)))


def gnn_aggregate_bwd(indptr_t, indices_t, edge_w_t, dY, dX, N, F, op, plan: Optional[Plan] = None, stream=None,
                      workspace=None, ldx=None, ldy=None, flags=0, max_slices=0) -> None:
    """dX = adjoint of the forward map, over the transposed graph (see include/gnnagg.h)."""
    _aggregate("gnn_aggregate_bwd", indptr_t, indices_t, edge_w_t, dY, dX, N, F, op, plan, stream, workspace, ldx, ldy, flags,
               max_slices)


def _row_stride(t: Optional[torch.Tensor]) -> int:
    if t is None or t.dim() != 2 or t.shape[0] <= 1:
        return 0
    if t.stride(1) != 1:
        raise ValueError("feature matrices must have unit column stride")
    return int(t.stride(0))


def _ap_opts(indptr, plan, stream, edge_ids, edge_width, ldv, lde, ldo, flags=0, max_slices=0) -> GnnApOpts:
    o = GnnApOpts()
    o.flags = int(flags)
    o.max_slices = int(max_slices)
    o.indptr_is_64 = 0 if indptr is None else _is64(indptr)
    o.edge_width = int(edge_width)
    o.ldv, o.lde, o.ldo = int(ldv), int(lde), int(ldo)
    if edge_ids is not None:
        if edge_ids.dtype != torch.int64:
            raise TypeError("edge_ids must be int64")
        o.edge_ids = _ptr(edge_ids)
    o.stream = _stream(stream)
    o.plan = plan.handle if plan is not None else None
    return o


def _edge_width(fE: Optional[torch.Tensor], d: int) -> int:
    if fE is None:
        return 0
    return 1 if (fE.dim() == 1 or fE.shape[1] == 1) and d != 1 else 0


def _f32(*tensors) -> None:
    for t in tensors:
        if t is not None and t.dtype != torch.float32:
            raise TypeError("the general primitive takes float32 features")


def gnn_ap_fwd(indptr, indices, fV, fE, fO, arg_e, N, d, binop, reduce, plan: Optional[Plan] = None, edge_ids=None,
               stream=None, flags=0, max_slices=0) -> None:
    """f_O[v] = reduce_e binop(f_V[u_e], f_E[e]) with any operator pair of Table 1 (see include/gnnagg.h).
    f_E may be [E, d] or [E] / [E, 1] (one scalar per edge)."""
    _f32(fV, fE, fO)
    if arg_e is not None and (arg_e.dtype != torch.int32 or not arg_e.is_contiguous()):
        raise TypeError("arg_e must be a contiguous int32 tensor")
    o = _ap_opts(indptr, plan, stream, edge_ids, _edge_width(fE, d), _row_stride(fV), _row_stride(fE) if fE is not None and fE.dim() == 2 else 0,
                 _row_stride(fO), flags, max_slices)
    _call_allocating("gnn_ap_fwd", lambda: load_library().gnn_ap_fwd(
        _ptr(indptr), _ptr(indices), _ptr(fV), _ptr(fE), _ptr(fO), _ptr(arg_e), int(N), int(d), int(binop), int(reduce),
        ctypes.byref(o)))


def gnn_ap_bwd_vertex(indptr_t, indices_t, dO, fE, dfV, N, d, binop, plan: Optional[Plan] = None, edge_ids=None,
                      stream=None) -> None:
    """Gradient with respect to f_V for the sum reducer, over the transposed graph (see include/gnnagg.h)."""
    _f32(dO, fE, dfV)
    o = _ap_opts(indptr_t, plan, stream, edge_ids, _edge_width(fE, d), _row_stride(dfV),
                 _row_stride(fE) if fE is not None and fE.dim() == 2 else 0, _row_stride(dO))
    _call_allocating("gnn_ap_bwd_vertex", lambda: load_library().gnn_ap_bwd_vertex(
        _ptr(indptr_t), _ptr(indices_t), _ptr(dO), _ptr(fE), _ptr(dfV), int(N), int(d), int(binop), ctypes.byref(o)))


def gnn_ap_bwd_vertex_arg(indices, arg_e, dO, fE, dfV, n_vertex_rows, N, d, binop, edge_ids=None, stream=None) -> None:
    """Gradient with respect to f_V for max / min: scatter to the winners (see include/gnnagg.h)."""
    _f32(dO, fE, dfV)
    o = _ap_opts(None, None, stream, edge_ids, _edge_width(fE, d), _row_stride(dfV),
                 _row_stride(fE) if fE is not None and fE.dim() == 2 else 0, _row_stride(dO))
    _check("gnn_ap_bwd_vertex_arg", load_library().gnn_ap_bwd_vertex_arg(
        _ptr(indices), _ptr(arg_e), _ptr(dO), _ptr(fE), _ptr(dfV), int(n_vertex_rows), int(N), int(d), int(binop),
        ctypes.byref(o)))


def gnn_ap_bwd_edge(indptr, indices, arg_e, fV, fE, dO, dfE, N, d, binop, plan: Optional[Plan] = None, edge_ids=None,
                    stream=None) -> None:
    """Gradient with respect to f_E, one row per edge (see include/gnnagg.h).  dfE has f_E's shape."""
    _f32(fV, fE, dO, dfE)
    o = _ap_opts(indptr, plan, stream, edge_ids, _edge_width(dfE, d), _row_stride(fV),
                 _row_stride(dfE) if dfE.dim() == 2 else 0, _row_stride(dO))
    _check("gnn_ap_bwd_edge", load_library().gnn_ap_bwd_edge(
        _ptr(indptr), _ptr(indices), _ptr(arg_e), _ptr(fV), _ptr(fE), _ptr(dO), _ptr(dfE), int(N), int(d), int(binop),
        ctypes.byref(o)))


def gnn_matmul_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load_library().gnn_matmul_workspace_bytes(int(M), int(N), int(K)))


def gnn_matmul(A, B, C, trans_a=False, trans_b=False, bias=None, relu=False, workspace=None, stream=None) -> None:
    """C = act(opA(A) @ opB(B) + bias) on the matrix cores (see include/gnnagg.h).  A, B, C are 2-D
    float32 tensors with unit column stride; shapes follow torch.matmul after the transposes."""
    _f32(A, B, C, bias)
    for t in (A, B, C):
        if t.dim() != 2 or (t.numel() > 0 and t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("matrices must be 2-D with unit column stride")
    M, K = (A.shape[1], A.shape[0]) if trans_a else (A.shape[0], A.shape[1])
    Kb, N = (B.shape[1], B.shape[0]) if trans_b else (B.shape[0], B.shape[1])
    if K != Kb or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    ld = lambda t: max(1, int(t.stride(0)) if t.shape[0] > 1 and t.numel() > 0 else int(t.shape[1]))  # noqa: E731
    _check("gnn_matmul", load_library().gnn_matmul(
        _ptr(A), ld(A), 1 if trans_a else 0, _ptr(B), ld(B), 1 if trans_b else 0, _ptr(C), ld(C), int(M), int(N), int(K),
        _ptr(bias), 1 if relu else 0, _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)))


def _dense(*tensors) -> None:
    for t in tensors:
        if t is not None and not t.is_contiguous():
            raise ValueError("the layer calls take dense (contiguous) tensors")


def gnn_sage_layer_saved_elems(N, F_in, F_out, order=0) -> int:
    return int(load_library().gnn_sage_layer_saved_elems(int(N), int(F_in), int(F_out), int(order)))


def gnn_sage_layer_workspace_bytes(N, F_in, F_out, relu=True, order=0) -> int:
    return int(load_library().gnn_sage_layer_workspace_bytes(int(N), int(F_in), int(F_out), 1 if relu else 0, int(order)))


GNN_LAYER_FORCE_PRODUCER_LAYOUT = 1
GNN_LAYER_NO_PRODUCER_LAYOUT = 2
GNN_LAYER_NO_GATE_FOLD = 4


def _layer_opts(indptr, plan, relu, order, stream, workspace=None, flags=0) -> GnnLayerOpts:
    o = GnnLayerOpts()
    o.flags = int(flags)
    o.indptr_is_64 = _is64(indptr)
    o.relu = 1 if relu else 0
    o.order = int(order)
    o.stream = _stream(stream)
    o.plan = plan.handle if plan is not None else None
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    return o


def gnn_sage_layer_fwd(indptr, indices, X, W, bias, saved, H, plan: Plan, relu=True, order=0, stream=None, flags=0) -> None:
    """H = act(aggregate(X) W + b), one GraphSAGE layer (see include/gnnagg.h)."""
    _f32(X, W, bias, saved, H)
    _dense(X, W, bias, saved, H)
    o = _layer_opts(indptr, plan, relu, order, stream, flags=flags)
    _call_allocating("gnn_sage_layer_fwd", lambda: load_library().gnn_sage_layer_fwd(
        _ptr(indptr), _ptr(indices), _ptr(X), _ptr(W), _ptr(bias), _ptr(saved), _ptr(H), int(X.shape[0]), int(W.shape[0]),
        int(W.shape[1]), ctypes.byref(o)))


def gnn_sage_layer_bwd(indptr_t, indices_t, X, W, saved, H, dH, dX, dW, db, plan: Plan, workspace, relu=True, order=0,
                       stream=None, flags=0) -> None:
    """Gradients of one layer over the transposed graph (see include/gnnagg.h)."""
    _f32(X, W, saved, H, dH, dX, dW, db)
    _dense(X, W, saved, H, dH, dX, dW, db)
    o = _layer_opts(indptr_t, plan, relu, order, stream, workspace, flags=flags)
    _call_allocating("gnn_sage_layer_bwd", lambda: load_library().gnn_sage_layer_bwd(
        _ptr(indptr_t), _ptr(indices_t), _ptr(X), _ptr(W), _ptr(saved), _ptr(H), _ptr(dH), _ptr(dX), _ptr(dW), _ptr(db),
        int(X.shape[0]), int(W.shape[0]), int(W.shape[1]), ctypes.byref(o)))


def gnn_csr_from_sorted_coo(dst_sorted: torch.Tensor, N: int, indptr_out: torch.Tensor, stream=None) -> None:
    st = load_library().gnn_csr_from_sorted_coo(_ptr(dst_sorted), int(dst_sorted.numel()), int(N), _ptr(indptr_out),
                                                _is64(indptr_out), _stream(stream))
    _check("gnn_csr_from_sorted_coo", st)


def gnn_transpose_csr(indptr, indices, edge_w, N, indptr_t, indices_t, perm=None, edge_w_t=None, stream=None) -> None:
    if indptr_t.dtype != indptr.dtype:
        raise TypeError("indptr_t must have the dtype of indptr")
    if perm is not None and perm.dtype != torch.int64:
        raise TypeError("perm must be int64")
    _call_allocating("gnn_transpose_csr", lambda: load_library().gnn_transpose_csr(
        _ptr(indptr), _ptr(indices), _ptr(edge_w), int(N), _is64(indptr), _ptr(indptr_t), _ptr(indices_t), _ptr(perm),
        _ptr(edge_w_t), _stream(stream)))


def gnn_validate_csr(indptr, indices, N, E, stream=None) -> int:
    """Returns the status (GNN_OK or GNN_ERR_INVALID_GRAPH); raises on other errors."""
    st = load_library().gnn_validate_csr(_ptr(indptr), _ptr(indices), int(N), int(E), _is64(indptr), _stream(stream))
    if st not in (GNN_OK, GNN_ERR_INVALID_GRAPH):
        raise GnnError("gnn_validate_csr", st)
    return st


def gnn_calib_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    st = load_library().gnn_calib_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream(stream))
    _check("gnn_calib_copy", st)


def gnn_calib_gather(table: torch.Tensor, n_lines: int, line_ids: torch.Tensor, out: torch.Tensor, stream=None) -> int:
    """Bare gather of 128-byte lines (see include/gnnagg.h); returns the number of lines one call fetches."""
    st = load_library().gnn_calib_gather(_ptr(table), int(n_lines), _ptr(line_ids), line_ids.numel(), _ptr(out), out.numel(),
                                         _stream(stream))
    _check("gnn_calib_gather", st)
    return line_ids.numel() // (1 << 20) // 16 * 16 * (1 << 20)
