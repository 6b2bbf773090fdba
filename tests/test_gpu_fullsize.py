"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times (default plans): outputs of sampled rows are recomputed one by one by the
oracle, and properties that hold at any size (all-ones invariant, adjoint
identity) are checked on the whole output."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import OP_CODE, assert_close

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]
DEV = torch.device("cuda:0")


def _sample_rows(deg: np.ndarray, seed: int, n_top=48, n_rand=3000, n_empty=16):
    rng = np.random.default_rng(seed)
    top = np.argsort(deg)[-n_top:]
    rnd = rng.choice(len(deg), size=min(n_rand, len(deg)), replace=False)
    empty = np.flatnonzero(deg == 0)[:n_empty]
    return np.unique(np.concatenate([top, rnd, empty])).astype(np.int64)


def _fullsize(name, f, op_name, weighted=False, dtype=torch.float32):
    print(f"[fullsize] {name} F={f} op={op_name}", flush=True)
    w_cfg = synth.WORKLOADS[name]
    el = synth.make_graph(name, device=DEV)
    assert (el.n, el.e) == (w_cfg["n"], w_cfg["e"])
    weights = synth.gcn_sym_edge_weights(el.dst, el.src, el.n) if weighted else None
    dg = gnn.build_device_graph(el.dst, el.src, el.n, edge_w=weights, indptr64=w_cfg["indptr64"])
    op = OP_CODE[op_name]
    n, e = el.n, el.e

    X = synth.normal_features(n, f, 1, device=DEV, dtype=dtype)
    dY = synth.normal_features(n, f, 2, device=DEV, dtype=dtype)
    Y = torch.full_like(X, float("nan"))
    dX = torch.full_like(dY, float("nan"))
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, X, Y, n, f, op, plan=dg.plan_fwd)
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t, dY, dX, n, f, op, plan=dg.plan_bwd)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y).all()) and bool(torch.isfinite(dX).all())
    # the same two calls from packed copies kept by the caller (widths of more than one line)
    Yp = dXp = None
    code = gnn.GNN_BF16 if dtype == torch.bfloat16 else gnn.GNN_F32
    if gnn.gnn_packed_bytes(n, f, code) > 0:
        buf = torch.empty(gnn.gnn_packed_bytes(n, f, code) // 4, dtype=torch.float32, device=DEV)
        Yp, dXp = torch.full_like(X, float("nan")), torch.full_like(dY, float("nan"))
        gnn.gnn_pack_rows(dg.indptr, dg.indices, X, buf, n, f, op, False, plan=dg.plan_fwd)
        gnn.gnn_aggregate_packed(dg.indptr, dg.indices, dg.edge_w, buf, Yp, n, f, op, False, plan=dg.plan_fwd)
        gnn.gnn_pack_rows(dg.indptr_t, dg.indices_t, dY, buf, n, f, op, True, plan=dg.plan_bwd)
        gnn.gnn_aggregate_packed(dg.indptr_t, dg.indices_t, dg.edge_w_t, buf, dXp, n, f, op, True, plan=dg.plan_bwd)
        torch.cuda.synchronize()
        del buf

    # explicit weights, bound to the plans as bench.py binds them: the long rows as source-blocked pieces
    Yb = dXb = None
    if weighted:
        dg.plan_fwd.bind_edge_weights(dg.edge_w)
        dg.plan_bwd.bind_edge_weights(dg.edge_w_t)
        Yb, dXb = torch.full_like(X, float("nan")), torch.full_like(dY, float("nan"))
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, X, Yb, n, f, op, plan=dg.plan_fwd)
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t, dY, dXb, n, f, op, plan=dg.plan_bwd)
        torch.cuda.synchronize()
        dg.plan_fwd.bind_edge_weights(None)
        dg.plan_bwd.bind_edge_weights(None)

    # adjoint identity on the whole output, fp64 dot products (holds at any size)
    lhs = (Y.double() * dY.double()).sum().item()
    rhs = (X.double() * dX.double()).sum().item()
    scale = (Y.double().abs() * dY.double().abs()).sum().item()
    assert abs(lhs - rhs) <= 1e-6 * scale, (lhs, rhs, scale)

    # all-ones features: SUM without weights returns the in-degree / out-degree exactly
    ones = torch.ones((n, 8), device=DEV)
    cnt = torch.empty_like(ones)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, ones, cnt, n, 8, gnn.GNN_SUM, plan=dg.plan_fwd)
    din_gpu = torch.bincount(el.dst.long(), minlength=n)
    assert torch.equal(cnt[:, 3].long(), din_gpu) and int(din_gpu.max()) < (1 << 24)
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, ones, cnt, n, 8, gnn.GNN_SUM, plan=dg.plan_bwd)
    assert torch.equal(cnt[:, 5].long(), torch.bincount(el.src.long(), minlength=n))

    # sampled rows against the oracle (inputs come from the generators, never from the HIP path)
    dst_h, src_h = synth.to_csr_numpy(el)
    indptr = oracle.csr_indptr(dst_h, n)
    din = np.diff(indptr)
    w_h = None if weights is None else weights.cpu().numpy()
    Xh = X.float().cpu().numpy()
    rows = _sample_rows(din, 7)
    dout = np.bincount(src_h, minlength=n)
    Yo, S = oracle.aggregate_fwd(indptr, src_h, Xh, op=op, w=w_h, dout=dout, rows=rows, nthreads=8, want_scale=True)
    assert_close(Y[torch.from_numpy(rows).to(DEV)], Yo, S, dtype == torch.bfloat16, f"{name} fwd rows")
    if Yp is not None:
        assert_close(Yp[torch.from_numpy(rows).to(DEV)], Yo, S, dtype == torch.bfloat16, f"{name} fwd rows from the packed copy")
    if Yb is not None:
        assert_close(Yb[torch.from_numpy(rows).to(DEV)], Yo, S, dtype == torch.bfloat16, f"{name} fwd rows with bound weights")
    del Xh
    indptr_t, indices_t, perm = oracle.transpose(indptr, src_h)
    rows_t = _sample_rows(np.diff(indptr_t), 8)
    wt_h = None if w_h is None else w_h[perm]
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, dY.float().cpu().numpy(), op=op, wt=wt_h, din=din, rows=rows_t,
                                   nthreads=8, want_scale=True)
    assert_close(dX[torch.from_numpy(rows_t).to(DEV)], dXo, St, dtype == torch.bfloat16, f"{name} bwd rows")
    if dXp is not None:
        assert_close(dXp[torch.from_numpy(rows_t).to(DEV)], dXo, St, dtype == torch.bfloat16, f"{name} bwd rows from the packed copy")
    if dXb is not None:
        assert_close(dXb[torch.from_numpy(rows_t).to(DEV)], dXo, St, dtype == torch.bfloat16, f"{name} bwd rows with bound weights")
    # the integer structure at full size, bit for bit
    assert np.array_equal(dg.indptr.cpu().numpy().astype(np.int64), indptr)
    assert np.array_equal(dg.indptr_t.cpu().numpy().astype(np.int64), indptr_t)
    assert np.array_equal(dg.indices_t.cpu().numpy(), indices_t)
    p = gnn.gnn_plan_default_params()
    bo, rp, ch, _ = dg.plan_fwd.export()
    obo, orp, och = oracle.plan(indptr, list(p.thresholds)[:p.n_thresholds], p.hub_chunk)
    assert np.array_equal(bo, obo) and np.array_equal(rp, orp) and np.array_equal(ch, och)


def test_fullsize_sparse_stack_f100():
    """2,449,029 vertices / 123,718,280 edges, F=100, MEAN: the configuration bench.py reports."""
    _fullsize("rmat_sparse_stack", 100, "mean")


def test_fullsize_sparse_stack_f256():
    _fullsize("rmat_sparse_stack", 256, "mean")


def test_fullsize_sparse_stack_f100_sage_gcn():
    """The aggregator of the paper's own runs (sum + own vector, over in-degree + 1), full size."""
    _fullsize("rmat_sparse_stack", 100, "sage")


def test_fullsize_dense_wide_f602():
    """232,965 vertices / 114,615,892 edges, F=602, MEAN."""
    _fullsize("rmat_dense_wide", 602, "mean")


def test_fullsize_weighted_narrow_f8():
    """132,534 vertices / 79,000,000 edges, F=8, explicit fp32 weights."""
    _fullsize("rmat_weighted_narrow", 8, "sum", weighted=True)


def test_fullsize_dense_wide_f256():
    """The hidden width of the dense-degree workload (232,965 vertices, F=256, MEAN)."""
    _fullsize("rmat_dense_wide", 256, "mean")


def test_fullsize_weighted_narrow_f64():
    """132,534 vertices / 79,000,000 edges, F=64, explicit fp32 weights."""
    _fullsize("rmat_weighted_narrow", 64, "sum", weighted=True)


def test_fullsize_weighted_narrow_f64_gcn_without_weights():
    """Symmetric normalisation derived from the degrees (no weight array), full size: the
    coefficients come from the plan's column counts, folded into the copy of the gathered rows."""
    _fullsize("rmat_weighted_narrow", 64, "gcn")


def test_fullsize_sparse_stack_f100_gcn_without_weights():
    _fullsize("rmat_sparse_stack", 100, "gcn")
