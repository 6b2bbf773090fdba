"""The capacity workload at full size: 111,059,956 vertices, 1,615,685,872 directed edges,
int64 row pointers, bf16 features of width 128 (about 150 GB of HBM in this test).

The oracle cannot produce the whole output (it would be 114 GB of fp64), so sampled rows
(the highest-degree rows, random rows, empty rows) are recomputed by the oracle on a
compacted sub-problem drawn from the generators' own data, and the properties that hold
at any size (all-ones invariant, adjoint identity) are checked on everything."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import assert_close

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]
DEV = torch.device("cuda:0")
F = 128


def _chunked_dot(a, b, chunk=1 << 22):
    tot = 0.0
    mag = 0.0
    for s in range(0, a.shape[0], chunk):
        x = a[s:s + chunk].double()
        y = b[s:s + chunk].double()
        tot += float((x * y).sum())
        mag += float((x.abs() * y.abs()).sum())
    return tot, mag


def _compact_rows(key_sorted, other, rows, n):
    """Edges whose (sorted) key is in `rows`, as a compact CSR over `rows` with `other`
    renumbered into 0..n_used-1.  Pure index plumbing on the generator's edge list."""
    rows_t = torch.from_numpy(rows).to(DEV)
    lo = torch.searchsorted(key_sorted, rows_t.to(key_sorted.dtype), right=False)
    hi = torch.searchsorted(key_sorted, rows_t.to(key_sorted.dtype), right=True)
    cnt = hi - lo
    indptr = torch.zeros(len(rows) + 1, dtype=torch.int64, device=DEV)
    indptr[1:] = torch.cumsum(cnt, 0)
    total = int(indptr[-1])
    # position list: for each sampled row its edge range
    owner = torch.repeat_interleave(torch.arange(len(rows), device=DEV), cnt)
    pos = lo[owner] + (torch.arange(total, device=DEV) - indptr[owner])
    nbr = other[pos].long()
    used, inv = torch.unique(nbr, return_inverse=True)
    return indptr.cpu().numpy(), inv.to(torch.int32).cpu().numpy(), used


def _sample(deg, seed, n_top=24, n_rand=2000, n_empty=8):
    rng = np.random.default_rng(seed)
    top = torch.topk(deg, n_top).indices.cpu().numpy()
    rnd = rng.choice(deg.numel(), size=n_rand, replace=False)
    empty = torch.nonzero(deg == 0)[:n_empty, 0].cpu().numpy()
    return np.unique(np.concatenate([top, rnd, empty])).astype(np.int64)


def test_capacity_fullsize_bf16_int64():
    print("[capacity] generating graph", flush=True)
    el = synth.make_graph("rmat_capacity", device=DEV)
    n, e = el.n, el.e
    assert (n, e) == (111059956, 1615685872)
    din = torch.bincount(el.dst, minlength=n)
    dout = torch.bincount(el.src, minlength=n)
    print("[capacity] building CSR, transpose, plans", flush=True)
    dg = gnn.build_device_graph(el.dst, el.src, n, indptr64=True)
    assert dg.indptr.dtype == torch.int64 and int(dg.indptr[-1]) == e

    print("[capacity] all-ones invariant", flush=True)
    ones = torch.ones((n, 8), device=DEV)
    cnt = torch.empty_like(ones)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, ones, cnt, n, 8, gnn.GNN_SUM, plan=dg.plan_fwd)
    assert int(din.max()) < (1 << 24) and torch.equal(cnt[:, 2].long(), din)
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, ones, cnt, n, 8, gnn.GNN_SUM, plan=dg.plan_bwd)
    assert torch.equal(cnt[:, 6].long(), dout)
    del ones, cnt

    print("[capacity] features", flush=True)
    X = synth.normal_features(n, F, 1, device=DEV, dtype=torch.bfloat16)
    dY = synth.normal_features(n, F, 2, device=DEV, dtype=torch.bfloat16)
    Y = torch.empty_like(X)
    dX = torch.empty_like(X)
    # the plan of the forward graph at full size, bit for bit (row pointers come from the generator's list)
    indptr_h = oracle.csr_indptr(el.dst.cpu().numpy(), n)
    assert np.array_equal(dg.indptr.cpu().numpy(), indptr_h)
    p = gnn.gnn_plan_default_params()
    bo, rp, ch, cc = dg.plan_fwd.export()
    obo, orp, och = oracle.plan(indptr_h, list(p.thresholds)[:p.n_thresholds], p.hub_chunk)
    assert np.array_equal(bo, obo) and np.array_equal(rp, orp) and np.array_equal(ch, och)
    assert np.array_equal(cc, dout.cpu().numpy().astype(np.int32))
    del indptr_h, rp, orp, cc

    rows_f = _sample(din, 5)
    rows_b = _sample(dout, 6)
    # (src, dst) sorted by (src, dst) for the backward sample: a stable sort of the canonical list by source
    order = torch.sort(el.src, stable=True).indices
    src_sorted = el.src[order]
    dst_by_src = el.dst[order]
    del order
    for op, oop in ((gnn.GNN_SUM, oracle.OP_SUM), (gnn.GNN_MEAN, oracle.OP_MEAN)):
        print(f"[capacity] op={op} forward/backward", flush=True)
        Y.fill_(float("nan")); dX.fill_(float("nan"))
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y, n, F, op, plan=dg.plan_fwd)
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, dY, dX, n, F, op, plan=dg.plan_bwd)
        torch.cuda.synchronize()
        # adjoint identity over all 14.2 G elements (bf16 outputs: each side carries one rounding per element)
        lhs, mag_l = _chunked_dot(Y, dY)
        rhs, mag_r = _chunked_dot(X, dX)
        assert abs(lhs - rhs) <= 2e-4 * max(mag_l, mag_r), (lhs, rhs, mag_l, mag_r)
        # sampled rows, forward
        ip, ix, used = _compact_rows(el.dst, el.src, rows_f, n)
        Yo, S = oracle.aggregate_fwd(ip, ix, X[used].float().cpu().numpy(), op=oop, nthreads=16, want_scale=True)
        assert_close(Y[torch.from_numpy(rows_f).to(DEV)], Yo, S, True, f"capacity fwd op={op}")
        # sampled rows, backward (MEAN needs din of the gathered vertices)
        ip, ix, used = _compact_rows(src_sorted, dst_by_src, rows_b, n)
        dXo, St = oracle.aggregate_bwd(ip, ix, dY[used].float().cpu().numpy(), op=oop, din=din[used].cpu().numpy(),
                                       nthreads=16, want_scale=True)
        assert_close(dX[torch.from_numpy(rows_b).to(DEV)], dXo, St, True, f"capacity bwd op={op}")
    print("[capacity] done", flush=True)
