"""numpy-facing wrappers around oracle.c (argument marshalling only).

Inputs are numpy arrays; floating-point inputs are taken as float32 (a bf16
workload passes its bf16-rounded values widened to float32, which is exact) and
every result is float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

OP_SUM, OP_MEAN, OP_GCN_SYM, OP_SAGE_GCN = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_SRC_AP = os.path.join(_HERE, "ap_oracle.c")
_SRC_LAYER = os.path.join(_HERE, "layer_oracle.c")
SOURCES = (_SRC, _SRC_AP, _SRC_LAYER)
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None
_lib_path = _LIB


def compile_c(src, out: str) -> None:
    srcs = [src] if isinstance(src, str) else list(src)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-std=c11",
                           "-Wall", "-Wextra", "-o", out, *srcs, "-lm"])


def build_oracle(force: bool = False) -> str:
    """Compile the oracle's C files with gcc (-O2, OpenMP, no fast-math, no contraction)."""
    newest = max(os.path.getmtime(p) for p in SOURCES)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        compile_c(list(SOURCES), _LIB)
    return _LIB


def _open(path: str):
    lib = ctypes.CDLL(path)
    lib.oracle_max_threads.restype = ctypes.c_int
    for name in ("oracle_aggregate_fwd", "oracle_aggregate_bwd", "oracle_csr_indptr",
                 "oracle_transpose", "oracle_plan", "oracle_ap_fwd", "oracle_ap_bwd", "oracle_matmul",
                 "oracle_sage_layer_fwd", "oracle_sage_layer_bwd"):
        if hasattr(lib, name):  # a mutated single-file build holds only its own functions
            getattr(lib, name).restype = ctypes.c_int
    return lib


def use_library(path: Optional[str]) -> None:
    """Point the wrappers at another build of oracle.c (the mutation tests
    load deliberately broken copies to show that the pins catch them);
    None restores the real one."""
    global _lib, _lib_path
    _lib = None
    _lib_path = _LIB if path is None else path


def _load():
    global _lib
    if _lib is None:
        if _lib_path == _LIB:
            build_oracle()
        _lib = _open(_lib_path)
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _aggregate(fn_name, indptr, indices, w, X, op, other_deg, rows, nthreads, want_scale):
    lib = _load()
    indptr = _i64(indptr)
    indices = _i32(indices)
    X = _f32(X)
    assert X.ndim == 2
    n = indptr.shape[0] - 1
    f = X.shape[1]
    # X may have a different number of rows than the CSR (a compacted sub-problem whose
    # indices were renumbered into X's rows); the arithmetic is the same.
    assert indices.shape[0] == indptr[-1]
    assert indices.size == 0 or (indices.min() >= 0 and indices.max() < X.shape[0])
    w = None if w is None else _f32(w)
    other_deg = None if other_deg is None else _i64(other_deg)
    rows_a = None if rows is None else _i64(rows)
    count = n if rows is None else rows_a.shape[0]
    Y = np.empty((count, f), dtype=np.float64)
    S = np.empty((count, f), dtype=np.float64) if want_scale else None
    rc = getattr(lib, fn_name)(
        _p(indptr), _p(indices), _p(w), _p(X), ctypes.c_int64(f), _p(Y), _p(S),
        ctypes.c_int64(n), ctypes.c_int64(f), ctypes.c_int(op), _p(other_deg),
        _p(rows_a), ctypes.c_int64(count), ctypes.c_int(nthreads))
    if rc != 0:
        raise ValueError(f"{fn_name} rejected its arguments (code {rc})")
    return (Y, S) if want_scale else Y


def aggregate_fwd(indptr, indices, X, op=OP_SUM, w=None, dout=None, rows=None,
                  nthreads: int = 1, want_scale: bool = False):
    """Y64 (and optionally the magnitude sums S) of the forward aggregation."""
    return _aggregate("oracle_aggregate_fwd", indptr, indices, w, X, op, dout, rows, nthreads, want_scale)


def aggregate_bwd(indptr_t, indices_t, dY, op=OP_SUM, wt=None, din=None, rows=None,
                  nthreads: int = 1, want_scale: bool = False):
    """dX64 of the backward aggregation over the transposed graph."""
    return _aggregate("oracle_aggregate_bwd", indptr_t, indices_t, wt, dY, op, din, rows, nthreads, want_scale)


def csr_indptr(dst_sorted, n: int) -> np.ndarray:
    lib = _load()
    dst_sorted = _i32(dst_sorted)
    indptr = np.empty(n + 1, dtype=np.int64)
    rc = lib.oracle_csr_indptr(_p(dst_sorted), ctypes.c_int64(dst_sorted.shape[0]), ctypes.c_int64(n), _p(indptr))
    if rc != 0:
        raise ValueError(f"oracle_csr_indptr: bad destination array (code {rc})")
    return indptr


def transpose(indptr, indices):
    """(indptr_t int64, indices_t int32, perm int64) of the transposed graph."""
    lib = _load()
    indptr = _i64(indptr)
    indices = _i32(indices)
    n = indptr.shape[0] - 1
    e = int(indptr[-1])
    indptr_t = np.empty(n + 1, dtype=np.int64)
    indices_t = np.empty(e, dtype=np.int32)
    perm = np.empty(e, dtype=np.int64)
    rc = lib.oracle_transpose(_p(indptr), _p(indices), ctypes.c_int64(n), _p(indptr_t), _p(indices_t), _p(perm))
    if rc != 0:
        raise ValueError(f"oracle_transpose failed (code {rc})")
    return indptr_t, indices_t, perm


def plan(indptr, thresholds, hub_chunk: int):
    """(bin_offsets int64[k+2], row_perm int32[N], chunks int64[n_chunks, 3])."""
    lib = _load()
    indptr = _i64(indptr)
    n = indptr.shape[0] - 1
    thr = _i64(thresholds)
    k = thr.shape[0]
    bin_offsets = np.empty(k + 2, dtype=np.int64)
    row_perm = np.empty(n, dtype=np.int32)
    nc = ctypes.c_int64(0)
    rc = lib.oracle_plan(_p(indptr), ctypes.c_int64(n), _p(thr), ctypes.c_int(k), ctypes.c_int64(hub_chunk),
                         _p(bin_offsets), _p(row_perm), None, ctypes.byref(nc))
    if rc != 0:
        raise ValueError(f"oracle_plan failed (code {rc})")
    chunks = np.empty((nc.value, 3), dtype=np.int64)
    rc = lib.oracle_plan(_p(indptr), ctypes.c_int64(n), _p(thr), ctypes.c_int(k), ctypes.c_int64(hub_chunk),
                         _p(bin_offsets), _p(row_perm), _p(chunks), ctypes.byref(nc))
    if rc != 0:
        raise ValueError(f"oracle_plan failed (code {rc})")
    return bin_offsets, row_perm, chunks


def blocked_layout(indptr, indices, thresholds, min_degree: int, hot_lines: int, block_lines: int, max_piece: int,
                   rest_min_count: int):
    """Source-blocked layout of the long rows (the reading of Section 4.2's source blocks taken for
    the GPU: only rows of at least `min_degree` edges are cut along blocks of sources), as a plain
    definition written with numpy sorts.

    rank[v]   position of v among the vertices ordered by descending occurrence count in `indices`,
              equal counts by ascending id
    block(r)  0 for r < hot_lines; the last block for r >= rest_begin = #{v: count[v] >= rest_min_count}
              (or hot_lines if that is larger); else 1 + (r - hot_lines) // block_lines
    rows      those of degree >= min_degree, numbered h = 0, 1, ... by ascending (bin, row id), the
              order of the plan's row permutation (bin = number of thresholds <= degree)
    edges     of those rows, ordered by (block of the source's rank, h, rank, CSR position)
    pieces    maximal runs of equal (block, h) in that order, cut every max_piece edges:
              (begin, length, slot, h); the pieces of row h get the slots rowbase[h], rowbase[h]+1, ...
              in that order
    Returns (ranks int32[E_b], epos uint32[E_b], pieces int32[P, 4], rowbase uint32[R + 1], rank int32[N])."""
    indptr = _i64(indptr)
    indices = _i64(indices)
    n = indptr.shape[0] - 1
    deg = np.diff(indptr)
    count = np.bincount(indices, minlength=n)
    order = np.lexsort((np.arange(n), -count))          # by descending count, then ascending id
    rank = np.empty(n, dtype=np.int64)
    rank[order] = np.arange(n)
    thr = np.asarray(thresholds, dtype=np.int64)
    bins = (deg[:, None] >= thr[None, :]).sum(axis=1)
    rows = np.flatnonzero(deg >= min_degree)
    rows = rows[np.lexsort((rows, bins[rows]))]
    rest_begin = max(int((count >= rest_min_count).sum()), min(hot_lines, n))
    hot = min(hot_lines, n)
    n_mid = -(-(rest_begin - hot) // block_lines)
    n_blocks = n_mid + 2
    e_h, e_rank, e_pos = [], [], []
    for h, v in enumerate(rows):
        pos = np.arange(indptr[v], indptr[v + 1])
        e_pos.append(pos)
        e_rank.append(rank[indices[pos]])
        e_h.append(np.full(pos.shape[0], h, dtype=np.int64))
    if not e_h:
        z = np.zeros(0, dtype=np.int32)
        return z, z.astype(np.uint32), np.zeros((0, 4), dtype=np.int32), np.zeros(0, dtype=np.uint32), rank.astype(np.int32)
    e_h, e_rank, e_pos = np.concatenate(e_h), np.concatenate(e_rank), np.concatenate(e_pos)
    blk = np.where(e_rank < hot, 0, np.where(e_rank >= rest_begin, n_blocks - 1, 1 + (e_rank - hot) // block_lines))
    o = np.lexsort((e_pos, e_rank, e_h, blk))
    e_h, e_rank, e_pos, blk = e_h[o], e_rank[o], e_pos[o], blk[o]
    pieces = []
    next_slot_in_row = np.zeros(len(rows), dtype=np.int64)
    pieces_of_row = np.zeros(len(rows), dtype=np.int64)
    i, total = 0, e_h.shape[0]
    runs = []
    while i < total:
        j = i
        while j < total and blk[j] == blk[i] and e_h[j] == e_h[i]:
            j += 1
        for b in range(i, j, max_piece):
            runs.append((b, min(max_piece, j - b), int(e_h[i])))
            pieces_of_row[e_h[i]] += 1
        i = j
    rowbase = np.concatenate(([0], np.cumsum(pieces_of_row)))
    for b, ln, h in runs:
        pieces.append((b, ln, rowbase[h] + next_slot_in_row[h], h))
        next_slot_in_row[h] += 1
    return (e_rank.astype(np.int32), e_pos.astype(np.uint32), np.asarray(pieces, dtype=np.int32).reshape(-1, 4),
            rowbase.astype(np.uint32), rank.astype(np.int32))


# ---------------------------------------------------------------- general primitive (Table 1)
BIN_ADD, BIN_SUB, BIN_MUL, BIN_DIV, BIN_COPY_LHS, BIN_COPY_RHS = range(6)
RED_SUM, RED_MAX, RED_MIN = range(3)


def _ap_common(indptr, indices, fV, fE, d, eid):
    indptr = _i64(indptr)
    indices = _i32(indices)
    fV = None if fV is None else _f32(fV)
    fE = None if fE is None else _f32(fE)
    if fE is not None and fE.ndim == 1:
        fE = fE.reshape(-1, 1)
    eid = None if eid is None else _i64(eid)
    ldv = 0 if fV is None else fV.shape[1]
    lde = 0 if fE is None else fE.shape[1]
    ewidth = d if fE is None else fE.shape[1]
    assert indices.shape[0] == indptr[-1]
    if fV is not None:
        assert fV.shape[1] == d
        assert indices.size == 0 or (indices.min() >= 0 and indices.max() < fV.shape[0])
    if fE is not None:
        rows = indices if eid is None else eid
        assert rows.size == 0 or (eid is None and fE.shape[0] >= indices.shape[0]) or \
            (eid is not None and eid.min() >= 0 and eid.max() < fE.shape[0])
    return indptr, indices, fV, fE, eid, ldv, lde, ewidth


def ap_fwd(indptr, indices, fV, fE, d, binop, reduce, eid=None):
    """(O float64[N, d], S float64[N, d]) for the sum reducer, (O, arg int64[N, d]) for max / min."""
    lib = _load()
    indptr, indices, fV, fE, eid, ldv, lde, ewidth = _ap_common(indptr, indices, fV, fE, d, eid)
    n = indptr.shape[0] - 1
    O = np.empty((n, d), dtype=np.float64)
    S = np.empty((n, d), dtype=np.float64) if reduce == RED_SUM else None
    arg = np.empty((n, d), dtype=np.int64) if reduce != RED_SUM else None
    rc = lib.oracle_ap_fwd(_p(indptr), _p(indices), _p(eid), _p(fV), ctypes.c_int64(ldv), _p(fE), ctypes.c_int64(lde),
                           ctypes.c_int64(ewidth), _p(O), _p(S), _p(arg), ctypes.c_int64(n), ctypes.c_int64(d),
                           ctypes.c_int(binop), ctypes.c_int(reduce))
    if rc != 0:
        raise ValueError(f"oracle_ap_fwd rejected its arguments (code {rc})")
    return O, (S if reduce == RED_SUM else arg)


def ap_bwd(indptr, indices, fV, fE, dO, d, binop, reduce, eid=None, arg=None, n_vertex_rows=None, n_edge_rows=None):
    """((dV, SV), (dE, SE)): gradients with respect to f_V and f_E and their magnitude sums."""
    lib = _load()
    indptr, indices, fV, fE, eid, ldv, lde, ewidth = _ap_common(indptr, indices, fV, fE, d, eid)
    n = indptr.shape[0] - 1
    dO = _f32(dO)
    assert dO.shape == (n, d)
    arg = None if arg is None else _i64(arg)
    nv = n_vertex_rows if n_vertex_rows is not None else (fV.shape[0] if fV is not None else n)
    ne = n_edge_rows if n_edge_rows is not None else (fE.shape[0] if fE is not None else indices.shape[0])
    dV = np.empty((nv, d), dtype=np.float64)
    SV = np.empty((nv, d), dtype=np.float64)
    dE = np.empty((ne, ewidth), dtype=np.float64)
    SE = np.empty((ne, ewidth), dtype=np.float64)
    rc = lib.oracle_ap_bwd(_p(indptr), _p(indices), _p(eid), _p(fV), ctypes.c_int64(ldv), _p(fE), ctypes.c_int64(lde),
                           ctypes.c_int64(ewidth), _p(dO), ctypes.c_int64(d), _p(arg), _p(dV), _p(SV), ctypes.c_int64(nv),
                           _p(dE), _p(SE), ctypes.c_int64(ne), ctypes.c_int64(n), ctypes.c_int64(d),
                           ctypes.c_int(binop), ctypes.c_int(reduce))
    if rc != 0:
        raise ValueError(f"oracle_ap_bwd rejected its arguments (code {rc})")
    return (dV, SV), (dE, SE)


# ---------------------------------------------------------------- one GraphSAGE layer
def matmul(A, B, trans_a=False, trans_b=False, bias=None, relu=False):
    """(C, S) float64: C = act(opA(A) @ opB(B) + bias), S = sum_k |a b| + |bias|."""
    lib = _load()
    A, B = _f32(A), _f32(B)
    M, K = (A.shape[1], A.shape[0]) if trans_a else A.shape
    Kb, N = (B.shape[1], B.shape[0]) if trans_b else B.shape
    assert K == Kb
    bias = None if bias is None else _f32(bias)
    C = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64)
    rc = lib.oracle_matmul(_p(A), ctypes.c_int64(A.shape[1]), ctypes.c_int(1 if trans_a else 0), _p(B),
                           ctypes.c_int64(B.shape[1]), ctypes.c_int(1 if trans_b else 0), _p(C), _p(S),
                           ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), _p(bias), ctypes.c_int(1 if relu else 0))
    if rc != 0:
        raise ValueError(f"oracle_matmul rejected its arguments (code {rc})")
    return C, S


def sage_layer_fwd(indptr, indices, X, W, bias=None, relu=True):
    """(Z, H, SH) float64 of one layer: aggregated input, output, magnitude sums of the output."""
    lib = _load()
    indptr, indices, X, W = _i64(indptr), _i32(indices), _f32(X), _f32(W)
    n, fi = X.shape
    fo = W.shape[1]
    assert W.shape[0] == fi and indptr.shape[0] == n + 1
    bias = None if bias is None else _f32(bias)
    Z = np.empty((n, fi), dtype=np.float64)
    H = np.empty((n, fo), dtype=np.float64)
    SH = np.empty((n, fo), dtype=np.float64)
    rc = lib.oracle_sage_layer_fwd(_p(indptr), _p(indices), _p(X), _p(W), _p(bias), _p(Z), _p(H), _p(SH),
                                   ctypes.c_int64(n), ctypes.c_int64(fi), ctypes.c_int64(fo), ctypes.c_int(1 if relu else 0))
    if rc != 0:
        raise ValueError(f"oracle_sage_layer_fwd failed (code {rc})")
    return Z, H, SH


def sage_layer_bwd(indptr, indices, X, W, H_saved, dH, relu=True):
    """{"dX": (value, scale), "dW": ..., "db": ...} float64 gradients of one layer."""
    lib = _load()
    indptr, indices, X, W, H_saved, dH = _i64(indptr), _i32(indices), _f32(X), _f32(W), _f32(H_saved), _f32(dH)
    n, fi = X.shape
    fo = W.shape[1]
    assert H_saved.shape == (n, fo) and dH.shape == (n, fo)
    out = {k: (np.empty(shape, dtype=np.float64), np.empty(shape, dtype=np.float64))
           for k, shape in (("dX", (n, fi)), ("dW", (fi, fo)), ("db", (fo,)))}
    rc = lib.oracle_sage_layer_bwd(_p(indptr), _p(indices), _p(X), _p(W), _p(H_saved), _p(dH),
                                   _p(out["dX"][0]), _p(out["dX"][1]), _p(out["dW"][0]), _p(out["dW"][1]),
                                   _p(out["db"][0]), _p(out["db"][1]),
                                   ctypes.c_int64(n), ctypes.c_int64(fi), ctypes.c_int64(fo), ctypes.c_int(1 if relu else 0))
    if rc != 0:
        raise ValueError(f"oracle_sage_layer_bwd failed (code {rc})")
    return out
