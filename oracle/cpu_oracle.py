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
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None
_lib_path = _LIB


def compile_c(src: str, out: str) -> None:
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                           "-Wall", "-Wextra", "-o", out, src, "-lm"])


def build_oracle(force: bool = False) -> str:
    """Compile oracle.c with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_c(_SRC, _LIB)
    return _LIB


def _open(path: str):
    lib = ctypes.CDLL(path)
    lib.oracle_max_threads.restype = ctypes.c_int
    for name in ("oracle_aggregate_fwd", "oracle_aggregate_bwd", "oracle_csr_indptr",
                 "oracle_transpose", "oracle_plan"):
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
