"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import (OP_CODE, assert_close, device_graph, host_csr, run_bwd, run_fwd, strict_relative_error)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _features(kind, n, f, seed, dtype=torch.float32):
    if kind == "uniform":
        return synth.uniform_features(n, f, seed, dtype=dtype)
    return synth.normal_features(n, f, seed, dtype=dtype)


def _check_both_directions(el, f, op_name, dtype=torch.float32, weights=None, indptr64=False, plan_params=None,
                           dist="normal", use_plan=True, seed=0, nthreads=8):
    """Forward and backward on one graph / width / op, whole output compared."""
    op = OP_CODE[op_name]
    bf16 = dtype == torch.bfloat16
    dg = device_graph(el, weights=weights, indptr64=indptr64, plan_params=plan_params)
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    din = np.diff(indptr)
    dout = np.diff(indptr_t)
    w = None if weights is None else weights.numpy()
    wt = None if w is None else w[perm]
    X = _features(dist, el.n, f, 1000 + seed, dtype)
    dY = _features(dist, el.n, f, 2000 + seed, dtype)
    plan_f = "default" if use_plan else None
    Y = run_fwd(dg, X.to(DEV), op, plan=plan_f)
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, w=w, dout=dout, nthreads=nthreads,
                                 want_scale=True)
    assert_close(Y, Yo, S, bf16, f"fwd {op_name} F={f}")
    dX = run_bwd(dg, dY.to(DEV), op, plan=plan_f)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, dY.float().numpy(), op=op, wt=wt, din=din,
                                   nthreads=nthreads, want_scale=True)
    assert_close(dX, dXo, St, bf16, f"bwd {op_name} F={f}")
    return strict_relative_error(Y, Yo, S), strict_relative_error(dX, dXo, St)


# ------------------------------------------------------------ the five workloads
def test_workload_er_tiny_full():
    """Tiny plumbing case at its full size: 4,096 vertices, 65,536 edges, F=64, SUM."""
    el = synth.make_graph("er_tiny")
    assert (el.n, el.e) == (4096, 65536)
    _check_both_directions(el, 64, "sum", dist="uniform")


@pytest.mark.parametrize("f", [602, 256])
def test_workload_dense_wide_scaled(f):
    """Dense-degree / wide-feature case (MEAN), graph scaled to 2% (mean degree ~490 kept)."""
    el = synth.make_graph("rmat_dense_wide", scale=0.02)
    _check_both_directions(el, f, "mean")


@pytest.mark.parametrize("f", [100, 256])
def test_workload_sparse_stack_scaled(f):
    """Sparse / medium-feature case (MEAN), graph scaled to 2%."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.02)
    _check_both_directions(el, f, "mean")


@pytest.mark.parametrize("f", [8, 64])
def test_workload_weighted_narrow_scaled(f):
    """Narrow-feature case with explicit fp32 GCN weights (SUM with weights), graph scaled to 2%."""
    el = synth.make_graph("rmat_weighted_narrow", scale=0.02)
    w = synth.gcn_sym_edge_weights(el.dst, el.src, el.n)
    _check_both_directions(el, f, "sum", weights=w)


@pytest.mark.parametrize("op_name", ["sum", "mean"])
def test_workload_capacity_scaled(op_name):
    """Capacity case at 0.05%: directed R-MAT, int64 row pointers, bf16 storage, F=128."""
    el = synth.make_graph("rmat_capacity", scale=0.0005)
    _check_both_directions(el, 128, op_name, dtype=torch.bfloat16, indptr64=True)


# -------------------------------------------------------------- shapes and ops
WIDTHS = [1, 2, 3, 4, 6, 8, 12, 30, 64, 100, 128, 130, 255, 256, 258, 602, 1030, 2052]


@pytest.mark.parametrize("f", WIDTHS)
def test_widths_f32(f):
    el = synth.make_graph("rmat_sparse_stack", scale=0.0008, seed=11)
    _check_both_directions(el, f, "mean", seed=f)


@pytest.mark.parametrize("f", [1, 2, 4, 7, 8, 24, 128, 136, 520, 1000])
def test_widths_bf16(f):
    el = synth.make_graph("rmat_sparse_stack", scale=0.0008, seed=12)
    _check_both_directions(el, f, "sum", dtype=torch.bfloat16, seed=f)


@pytest.mark.parametrize("op_name", ["sum", "mean", "gcn", "sage"])
@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("use_plan", [False, True])
def test_ops_weights_plan(op_name, weighted, use_plan):
    if not use_plan and (op_name == "gcn" and not weighted):
        pytest.skip("weight-less GCN_SYM needs a plan (tested in test_errors)")
    el = synth.make_graph("rmat_sparse_stack", scale=0.001, seed=21)
    # properly directed graph: drop a seeded half of the edges so that CSR != CSC
    keep = torch.from_numpy(np.random.default_rng(3).random(el.e) < 0.5)
    el = synth.EdgeList(el.n, el.src[keep], el.dst[keep], el.meta)
    w = None
    if weighted:
        w = torch.from_numpy(np.random.default_rng(4).uniform(0.1, 2.0, el.e).astype(np.float32))
    if not use_plan and op_name in ("mean", "sage"):
        # the backward pass of these ops needs a plan; check forward only
        dg = device_graph(el, weights=w, with_plans=False)
        indptr, indices, *_ = host_csr(el)
        X = synth.normal_features(el.n, 40, 5)
        Y = run_fwd(dg, X.to(DEV), OP_CODE[op_name], plan=None)
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.numpy(), op=OP_CODE[op_name],
                                     w=None if w is None else w.numpy(), want_scale=True)
        assert_close(Y, Yo, S, False, f"fwd {op_name} no plan")
        return
    _check_both_directions(el, 40, op_name, weights=w, use_plan=use_plan)


PLAN_VARIANTS = {
    "default": None,
    "all_rows_are_hubs": ([], 7),
    "all_rows_are_hubs_big_chunk": ([], 1 << 20),
    "one_bin_no_hub": ([], 0),
    "two_bins_hub_at_3": ([3], 5),
    "fine_bins_no_hub": ([1, 2, 3, 5, 9, 17, 33, 65, 129, 257, 513, 1025, 2049, 4097, 8193], 0),
    "wave_rows_only": ([64], 0),
    "hub_at_64": ([1, 8, 64], 64),
}


@pytest.mark.parametrize("variant", list(PLAN_VARIANTS))
@pytest.mark.parametrize("f", [8, 100, 602])
def test_every_kernel_family_gives_the_same_answer(variant, f):
    """One owner per output row means scheduling cannot change the result:
    route the rows through each kernel family by moving the bin thresholds."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.002, seed=31)
    pv = PLAN_VARIANTS[variant]
    params = None if pv is None else gnn.make_plan_params(*pv)
    _check_both_directions(el, f, "mean", plan_params=params)
    _check_both_directions(el, f, "gcn", plan_params=params)
    _check_both_directions(el, f, "sage", plan_params=params)


@pytest.mark.parametrize("f,dtype", [(64, torch.float32), (256, torch.float32), (640, torch.float32),
                                     (160, torch.float32), (128, torch.bfloat16), (1024, torch.bfloat16)])
@pytest.mark.parametrize("hubs", [False, True])
def test_column_slices_over_xcds_on_and_off(f, dtype, hubs):
    """Line-aligned rows are gathered slice by slice (one slice per XCD); with the
    slicing switched off the same rows go through the whole-row path.  Both must
    match the oracle, with and without hub rows cut into pieces."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.004, seed=71)
    dg = device_graph(el, plan_params=gnn.make_plan_params([1, 4, 32], 48) if hubs else None)
    indptr, indices, *_ = host_csr(el)
    X = synth.normal_features(el.n, f, 9, dtype=dtype)
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=oracle.OP_MEAN, nthreads=8, want_scale=True)
    Xd = X.to(DEV)
    assert Xd.data_ptr() % 128 == 0
    outs = []
    for flags, max_slices in ((0, 0), (0, 8), (0, 2), (gnn.GNN_FLAG_NO_COLUMN_SLICES, 0)):
        Y = torch.full_like(Xd, float("nan"))
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, gnn.GNN_MEAN, plan=dg.plan_fwd, flags=flags,
                              max_slices=max_slices)
        torch.cuda.synchronize()
        assert_close(Y, Yo, S, dtype == torch.bfloat16, f"slices flags={flags} max={max_slices} F={f}")
        outs.append(Y)


@pytest.mark.parametrize("f,max_slices", [(4160, 2), (8160, 4), (8192, 2), (4100, 2)])
def test_very_wide_rows_take_many_sliced_launches(f, max_slices):
    """Rows of more than 64 lines with few slices per launch: 65 ... 128 launches plus a dense tail
    (the launch list once had room for 64)."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.0004, seed=72)
    dg = device_graph(el, plan_params=gnn.make_plan_params([1, 4, 32], 48))
    indptr, indices, *_ = host_csr(el)
    X = synth.normal_features(el.n, f, 10)
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.numpy(), op=oracle.OP_MEAN, nthreads=8, want_scale=True)
    Xd = X.to(DEV)
    for flags in (0, gnn.GNN_FLAG_FORCE_PADDED_COPY):
        Y = torch.full_like(Xd, float("nan"))
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, gnn.GNN_MEAN, plan=dg.plan_fwd, flags=flags,
                              max_slices=max_slices)
        torch.cuda.synchronize()
        assert_close(Y, Yo, S, False, f"wide rows F={f} max_slices={max_slices} flags={flags}")


@pytest.mark.parametrize("f,dtype", [(100, torch.float32), (602, torch.float32), (30, torch.float32), (7, torch.float32),
                                     (129, torch.float32), (2052, torch.float32), (100, torch.bfloat16),
                                     (602, torch.bfloat16), (9, torch.bfloat16), (1000, torch.bfloat16)])
@pytest.mark.parametrize("hubs", [False, True])
def test_padded_copy_route(f, dtype, hubs):
    """Widths whose rows are not whole 128-byte lines are gathered from a plan-owned padded
    copy (forced here; automatic for large matrices).  Loads run past column F into the
    padding, stores must not: the output is poisoned and checked column by column."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.003, seed=81)
    params = gnn.make_plan_params([2, 16], 24) if hubs else None
    dg = device_graph(el, plan_params=params)
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    X = synth.normal_features(el.n, f, 10, dtype=dtype)
    bf16 = dtype == torch.bfloat16
    for op, oop in ((gnn.GNN_MEAN, oracle.OP_MEAN), (gnn.GNN_GCN_SYM, oracle.OP_GCN_SYM), (gnn.GNN_SAGE_GCN, oracle.OP_SAGE_GCN)):
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=oop, dout=np.diff(indptr_t), nthreads=8,
                                     want_scale=True)
        dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=oop, din=np.diff(indptr), nthreads=8,
                                       want_scale=True)
        # output with a wider stride: the columns between F and ld must stay untouched
        ld = f + 5
        out = torch.full((el.n, ld), float("nan"), dtype=dtype, device=DEV)
        Y = out[:, :f]
        Xd = X.to(DEV)
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, op, plan=dg.plan_fwd,
                              flags=gnn.GNN_FLAG_FORCE_PADDED_COPY, ldy=ld)
        torch.cuda.synchronize()
        assert_close(Y, Yo, S, bf16, f"padded fwd F={f} op={op}")
        assert torch.isnan(out[:, f:]).all()
        out.fill_(float("nan"))
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, Y, el.n, f, op, plan=dg.plan_bwd,
                              flags=gnn.GNN_FLAG_FORCE_PADDED_COPY, ldy=ld)
        torch.cuda.synchronize()
        assert_close(Y, dXo, St, bf16, f"padded bwd F={f} op={op}")
        assert torch.isnan(out[:, f:]).all()


# -------------------------------------------------------------- integer parts
@pytest.mark.parametrize("name,scale,ip64", [("er_tiny", 1.0, False), ("rmat_sparse_stack", 0.02, False),
                                             ("rmat_dense_wide", 0.01, True), ("rmat_capacity", 0.0005, True)])
def test_csr_and_transpose_bit_exact(name, scale, ip64):
    el = synth.make_graph(name, scale=scale)
    w = torch.from_numpy(np.random.default_rng(1).random(el.e).astype(np.float32))
    dg = device_graph(el, weights=w, indptr64=ip64, want_perm=True, with_plans=False)
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    assert np.array_equal(dg.indptr.cpu().numpy().astype(np.int64), indptr)
    assert np.array_equal(dg.indptr_t.cpu().numpy().astype(np.int64), indptr_t)
    assert np.array_equal(dg.indices_t.cpu().numpy(), indices_t)
    assert np.array_equal(dg.perm.cpu().numpy(), perm)
    assert np.array_equal(dg.edge_w_t.cpu().numpy(), w.numpy()[perm])
    assert gnn.gnn_validate_csr(dg.indptr, dg.indices, el.n, el.e) == gnn.GNN_OK
    assert gnn.gnn_validate_csr(dg.indptr_t, dg.indices_t, el.n, el.e) == gnn.GNN_OK


@pytest.mark.parametrize("variant", list(PLAN_VARIANTS))
def test_plan_bit_exact(variant):
    el = synth.make_graph("rmat_sparse_stack", scale=0.02, seed=41)
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    pv = PLAN_VARIANTS[variant]
    if pv is None:
        p = gnn.gnn_plan_default_params()
        thr, chunk = list(p.thresholds)[:p.n_thresholds], p.hub_chunk
        params = None
    else:
        thr, chunk = pv
        params = gnn.make_plan_params(thr, chunk)
    dg = device_graph(el, plan_params=params)
    for plan, ip, ix in ((dg.plan_fwd, indptr, indices), (dg.plan_bwd, indptr_t, indices_t)):
        bo, rp, ch, cc = plan.export()
        obo, orp, och = oracle.plan(ip, thr, chunk)
        assert np.array_equal(bo, obo)
        assert np.array_equal(rp, orp)
        assert np.array_equal(ch, och)
        assert np.array_equal(cc, np.bincount(ix, minlength=el.n).astype(np.int32))


def test_gather_share_of_the_most_gathered_vertices():
    """The plan's bucket histogram answers 'which share of the gathers goes to the K
    most-gathered vertices' to within the bucket width (12 %)."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.05, seed=91)
    dg = device_graph(el)
    counts = np.sort(np.bincount(el.src.numpy(), minlength=el.n))[::-1].astype(np.float64)
    for k in (1, 10, 300, 4096, 32768, el.n, 10 * el.n):
        exact = counts[:k].sum() / el.e
        got = dg.plan_fwd.gather_share(k)
        assert abs(got - exact) <= 0.02 + 0.06 * exact, (k, got, exact)
    assert dg.plan_fwd.gather_share(0) == 0.0


# ------------------------------------------------------------------ edge cases
def test_empty_and_degenerate_inputs():
    dev = torch.device(DEV)
    # N == 0 and F == 0 are no-ops
    z32 = torch.zeros(1, dtype=torch.int32, device=dev)
    e = torch.zeros(0, dtype=torch.int32, device=dev)
    x0 = torch.zeros((0, 4), device=dev)
    gnn.gnn_aggregate_fwd(z32, e, None, x0, x0.clone(), 0, 4, gnn.GNN_SUM)
    # graph without edges: every op writes zeros over a poisoned output
    n = 300
    el = synth.EdgeList(n, torch.zeros(0, dtype=torch.int32), torch.zeros(0, dtype=torch.int32))
    dg = device_graph(el)
    X = synth.normal_features(n, 12, 1).to(dev)
    for op in (gnn.GNN_SUM, gnn.GNN_MEAN, gnn.GNN_GCN_SYM):
        assert not run_fwd(dg, X, op).any()
        assert not run_bwd(dg, X, op).any()
        assert not run_fwd(dg, X, gnn.GNN_SUM, plan=None).any()
    # the GraphSAGE-GCN aggregator of an edgeless graph is the vertex's own vector (divided by 0 + 1)
    assert torch.equal(run_fwd(dg, X, gnn.GNN_SAGE_GCN), X) and torch.equal(run_bwd(dg, X, gnn.GNN_SAGE_GCN), X)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X[:, :0], X[:, :0].clone(), n, 0, gnn.GNN_SUM)
    # one vertex with a self-loop, and a multigraph with duplicates and self-loops
    el = synth.EdgeList(1, torch.zeros(1, dtype=torch.int32), torch.zeros(1, dtype=torch.int32))
    _check_both_directions(el, 5, "mean")
    el = synth.small_random_multigraph(37, 500, 3)
    for op_name in ("sum", "mean", "gcn", "sage"):
        _check_both_directions(el, 9, op_name)
    # a star: one row with N-1 neighbours, N-1 rows with one
    n = 5000
    leaves = torch.arange(1, n, dtype=torch.int32)
    zeros = torch.zeros(n - 1, dtype=torch.int32)
    el = synth.EdgeList(n, torch.cat([leaves, zeros]), torch.cat([zeros, leaves]))
    _check_both_directions(el, 100, "mean")
    _check_both_directions(el, 100, "gcn", plan_params=gnn.make_plan_params([64], 256))
    _check_both_directions(el, 100, "sage", plan_params=gnn.make_plan_params([64], 256))


def test_strided_and_misaligned_rows():
    """ld > F, and base pointers / strides that only allow 8- or 4-byte loads."""
    dev = torch.device(DEV)
    el = synth.make_graph("rmat_sparse_stack", scale=0.001, seed=51)
    dg = device_graph(el)
    indptr, indices, *_ = host_csr(el)
    f = 100
    for ld, off in ((128, 0), (102, 2), (101, 1), (100, 3)):
        buf = synth.normal_features(el.n, ld + 4, 7).to(dev)
        flat = buf.view(-1)
        X = torch.as_strided(flat, (el.n, f), (ld, 1), storage_offset=off)
        out = torch.full((el.n * ld + 8,), float("nan"), device=dev)
        Y = torch.as_strided(out, (el.n, f), (ld, 1), storage_offset=off)
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y, el.n, f, gnn.GNN_MEAN, plan=dg.plan_fwd, ldx=ld, ldy=ld)
        torch.cuda.synchronize()
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.cpu().numpy(), op=oracle.OP_MEAN, want_scale=True)
        assert_close(Y, Yo, S, False, f"ld={ld} off={off}")
        if ld > f:  # the padding columns must stay untouched
            pad = torch.as_strided(out, (el.n - 1, ld - f), (ld, 1), storage_offset=off + f)
            assert torch.isnan(pad).all()


def test_errors():
    dev = torch.device(DEV)
    el = synth.make_graph("er_tiny")
    dg = device_graph(el)
    X = synth.uniform_features(el.n, 8, 1).to(dev)
    Y = torch.empty_like(X)

    def status(fn, *a, **k):
        with pytest.raises(gnn.GnnError) as ei:
            fn(*a, **k)
        return ei.value.status

    assert status(gnn.gnn_aggregate_fwd, dg.indptr, dg.indices, None, X, Y, el.n, 8, 7) == gnn.GNN_ERR_INVALID_ARG
    assert status(gnn.gnn_aggregate_fwd, dg.indptr, dg.indices, None, X, Y, -1, 8, 0) == gnn.GNN_ERR_INVALID_ARG
    assert status(gnn.gnn_aggregate_fwd, dg.indptr, dg.indices, None, X, Y, el.n, 8, 0, ldx=4) == gnn.GNN_ERR_INVALID_ARG
    assert status(gnn.gnn_aggregate_fwd, dg.indptr, dg.indices, None, X, Y, el.n + 1, 8, 0, plan=dg.plan_fwd) == gnn.GNN_ERR_INVALID_ARG
    assert status(gnn.gnn_aggregate_bwd, dg.indptr_t, dg.indices_t, None, X, Y, el.n, 8, gnn.GNN_MEAN) == gnn.GNN_ERR_UNSUPPORTED
    assert status(gnn.gnn_aggregate_fwd, dg.indptr, dg.indices, None, X, Y, el.n, 8, gnn.GNN_GCN_SYM) == gnn.GNN_ERR_UNSUPPORTED
    assert status(gnn.gnn_aggregate_bwd, dg.indptr_t, dg.indices_t, None, X, Y, el.n, 8, gnn.GNN_SAGE_GCN) == gnn.GNN_ERR_UNSUPPORTED
    assert status(gnn.gnn_plan_create, dg.indptr, dg.indices, el.n, gnn.make_plan_params([4, 2], 0)) == gnn.GNN_ERR_INVALID_ARG
    # a workspace that is too small is rejected, one that is large enough is used
    params = gnn.make_plan_params([8], 4)
    dg2 = device_graph(el, plan_params=params)
    need = dg2.plan_fwd.workspace_bytes(8)
    assert need > 0
    small = torch.empty(need // 4 - 1, dtype=torch.float32, device=dev)
    assert status(gnn.gnn_aggregate_fwd, dg2.indptr, dg2.indices, None, X, Y, el.n, 8, 0, plan=dg2.plan_fwd,
                  workspace=small) == gnn.GNN_ERR_INVALID_ARG
    big = torch.empty(need // 4, dtype=torch.float32, device=dev)
    gnn.gnn_aggregate_fwd(dg2.indptr, dg2.indices, None, X, Y, el.n, 8, 0, plan=dg2.plan_fwd, workspace=big)
    Y2 = run_fwd(dg, X, 0)
    torch.cuda.synchronize()
    assert torch.allclose(Y, Y2, rtol=1e-4, atol=1e-5)
    # broken graphs are reported by the validator
    bad = dg.indices.clone(); bad[5] = el.n
    assert gnn.gnn_validate_csr(dg.indptr, bad, el.n, el.e) == gnn.GNN_ERR_INVALID_GRAPH
    badp = dg.indptr.clone(); badp[10] = badp[11] + 1
    assert gnn.gnn_validate_csr(badp, dg.indices, el.n, el.e) == gnn.GNN_ERR_INVALID_GRAPH


def test_stream_and_repeatability():
    """Runs on a side stream, twice: results are bit-identical (no atomics, fixed reduction order)."""
    dev = torch.device(DEV)
    el = synth.make_graph("rmat_sparse_stack", scale=0.004, seed=61)
    dg = device_graph(el, plan_params=gnn.make_plan_params([1, 4, 16, 64, 256], 128))
    X = synth.normal_features(el.n, 100, 3).to(dev)
    s = torch.cuda.Stream()
    outs = []
    for _ in range(2):
        Y = torch.empty_like(X)
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y, el.n, 100, gnn.GNN_MEAN, plan=dg.plan_fwd)
        s.synchronize()
        outs.append(Y)
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("seed", range(40))
def test_randomised_shapes_and_options(seed):
    """Seeded random draws over graph shape, width, dtype, op, weights, bin thresholds, hub
    piece size, row strides, base offsets and the layout switches; every draw must match the
    oracle in both directions."""
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 6000))
    e = int(rng.integers(0, 40 * n + 1))
    kind = rng.choice(["multi", "rmat", "star"])
    if kind == "multi" or n < 64:
        el = synth.small_random_multigraph(n, max(e, 1), seed) if e > 0 else synth.EdgeList(
            n, torch.zeros(0, dtype=torch.int32), torch.zeros(0, dtype=torch.int32))
    elif kind == "rmat":
        e = min(e - e % 2, n * (n - 1) // 4 * 2)
        el = synth.rmat_symmetric(n, max(e, 2), (0.57, 0.19, 0.19, 0.05), seed)
    else:
        leaves = torch.arange(1, n, dtype=torch.int32)
        zeros = torch.zeros(n - 1, dtype=torch.int32)
        el = synth.EdgeList(n, torch.cat([leaves, zeros]), torch.cat([zeros, leaves]))
    f = int(rng.choice([1, 2, 3, 5, 8, 17, 32, 33, 64, 96, 100, 128, 160, 255, 256, 288, 602, 640, 1024, 1100]))
    dtype = torch.bfloat16 if rng.random() < 0.35 else torch.float32
    op_name = str(rng.choice(["sum", "mean", "gcn", "sage"]))
    weights = None
    if rng.random() < 0.4 and el.e > 0:
        weights = torch.from_numpy(rng.uniform(0.1, 2.0, el.e).astype(np.float32))
    k = int(rng.integers(0, 6))
    thr = sorted(set(int(t) for t in rng.integers(1, 200, size=k)))
    params = gnn.make_plan_params(thr, int(rng.choice([0, 3, 16, 64, 1024])))
    flags = int(rng.choice([0, gnn.GNN_FLAG_FORCE_PADDED_COPY, gnn.GNN_FLAG_FORCE_PADDED_COPY, gnn.GNN_FLAG_NO_COLUMN_SLICES,
                            gnn.GNN_FLAG_NO_PADDED_COPY]))
    flags |= int(rng.choice([0, 0, gnn.GNN_FLAG_NO_SLICE_TABLES, gnn.GNN_FLAG_NO_RANK_ORDER, gnn.GNN_FLAG_FORCE_COLD_HINTS,
                             gnn.GNN_FLAG_NO_COLD_HINTS]))
    max_slices = int(rng.choice([0, 0, 2, 4, 8]))
    ld = f + int(rng.choice([0, 0, 1, 3, 32, 96]))
    off = int(rng.choice([0, 0, 1, 4, 32]))

    op = OP_CODE[op_name]
    bf16 = dtype == torch.bfloat16
    dg = device_graph(el, weights=weights, plan_params=params)
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    w = None if weights is None else weights.numpy()
    wt = None if w is None else w[perm]
    what = f"seed={seed} n={el.n} e={el.e} f={f} {dtype} {op_name} w={w is not None} thr={thr} flags={flags} S<={max_slices} ld={ld} off={off}"
    print(what, flush=True)

    def strided(seed_):
        base = synth.normal_features(el.n, ld + 1, seed_, dtype=dtype).to(DEV).view(-1)
        need = off + (el.n - 1) * ld + f
        assert base.numel() >= need
        return base, torch.as_strided(base, (el.n, f), (ld, 1), storage_offset=off)

    _, X = strided(1)
    _, dY = strided(2)
    out_buf = torch.full((el.n * ld + off + 8,), float("nan"), dtype=dtype, device=DEV)
    out = torch.as_strided(out_buf, (el.n, f), (ld, 1), storage_offset=off)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, X, out, el.n, f, op, plan=dg.plan_fwd, ldx=ld, ldy=ld,
                          flags=flags, max_slices=max_slices)
    torch.cuda.synchronize()
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().cpu().numpy(), op=op, w=w, dout=dout, nthreads=8, want_scale=True)
    assert_close(out, Yo, S, bf16, "fwd " + what)
    written = torch.zeros(out_buf.numel(), dtype=torch.bool, device=DEV)
    torch.as_strided(written, (el.n, f), (ld, 1), storage_offset=off).fill_(True)
    assert torch.isnan(out_buf[~written]).all(), "stores outside the output rows: " + what
    out_buf.fill_(float("nan"))
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t, dY, out, el.n, f, op, plan=dg.plan_bwd, ldx=ld, ldy=ld,
                          flags=flags, max_slices=max_slices)
    torch.cuda.synchronize()
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, dY.float().cpu().numpy(), op=op, wt=wt, din=din, nthreads=8,
                                   want_scale=True)
    assert_close(out, dXo, St, bf16, "bwd " + what)
    assert torch.isnan(out_buf[~written]).all(), "stores outside the output rows: " + what


@pytest.mark.parametrize("f,ld", [(47, 48), (5, 8), (101, 104)])
def test_padded_rows_flag_allows_wide_loads(f, ld):
    """With GNN_FLAG_PADDED_ROWS the padding of the gathered rows may be read (and must be ignored):
    it is filled with NaN here."""
    el = synth.rmat_symmetric(3000, 60000, (0.57, 0.19, 0.19, 0.05), 2)
    dg = device_graph(el, plan_params=gnn.make_plan_params([4, 32], 64))
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    buf = torch.full((el.n, ld), float("nan"), device=DEV)
    X = synth.normal_features(el.n, f, 3)
    buf[:, :f] = X.to(DEV)
    out = torch.full((el.n, ld), float("nan"), device=DEV)
    for op_name in ("sum", "sage"):
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, buf[:, :f], out[:, :f], el.n, f, OP_CODE[op_name], plan=dg.plan_fwd,
                              ldx=ld, ldy=ld, flags=gnn.GNN_FLAG_PADDED_ROWS)
        torch.cuda.synchronize()
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.numpy(), op=OP_CODE[op_name], nthreads=8, want_scale=True)
        assert_close(out[:, :f], Yo, S, False, f"padded rows {op_name} F={f}")
        assert torch.isnan(out[:, f:]).all(), "the output padding must stay untouched"


@pytest.mark.parametrize("case", ["er_tiny", "hubs_padded_sliced"])
def test_graph_capture_replays_match_eager(case):
    """The hot calls allocate nothing once the plan is prepared and record no memset, so a step can
    be captured into a HIP graph; every replay (with eager work between replays) must reproduce
    the eager result bit for bit."""
    if case == "er_tiny":
        el, f, params, flags, max_slices = synth.make_graph("er_tiny"), 64, None, 0, 0
    else:
        el = synth.rmat_symmetric(20000, 600000, (0.57, 0.19, 0.19, 0.05), 3)
        f, params, flags, max_slices = 100, gnn.make_plan_params([4, 32, 256], 128), gnn.GNN_FLAG_FORCE_PADDED_COPY, 4
    dg = device_graph(el, plan_params=params)
    op = gnn.GNN_MEAN
    X = synth.normal_features(el.n, f, 1).to(DEV)
    dY = synth.normal_features(el.n, f, 2).to(DEV)
    Y, dX = torch.empty_like(X), torch.empty_like(dY)

    def step():
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y, el.n, f, op, plan=dg.plan_fwd, flags=flags, max_slices=max_slices)
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, dY, dX, el.n, f, op, plan=dg.plan_bwd, flags=flags, max_slices=max_slices)

    step()  # first use: plan-owned buffers are grown here, outside the capture
    torch.cuda.synchronize()
    want_Y, want_dX = Y.clone(), dX.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        Y.fill_(float("nan"))
        dX.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, want_Y) and torch.equal(dX, want_dX), f"replay {rep}"
        # eager work between the replays, new inputs for the next one
        X.mul_(1.5)
        dY.add_(0.25)
        step()
        torch.cuda.synchronize()
        want_Y, want_dX = Y.clone(), dX.clone()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("f", [5, 64, 100, 256])
def test_cold_hints_do_not_change_results(f, dtype):
    """Sources flagged as cold are fetched with non-temporal loads; forced here on a small graph
    (a quarter of the vertices stays warm), every layout, both directions, bit-identical output."""
    el = synth.rmat_symmetric(6000, 150000, (0.57, 0.19, 0.19, 0.05), 8)
    bf16 = dtype == torch.bfloat16
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    X = synth.normal_features(el.n, f, 3, dtype=dtype)
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=OP_CODE["mean"], nthreads=8, want_scale=True)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=OP_CODE["mean"], din=np.diff(indptr), nthreads=8,
                                   want_scale=True)
    Xd = X.to(DEV)
    for layout_flags, max_slices in ((0, 0), (gnn.GNN_FLAG_FORCE_PADDED_COPY, 8), (gnn.GNN_FLAG_NO_PADDED_COPY, 2)):
        outs = []
        for hint in (gnn.GNN_FLAG_NO_COLD_HINTS, gnn.GNN_FLAG_FORCE_COLD_HINTS):
            dg = device_graph(el, plan_params=gnn.make_plan_params([4, 32, 256], 64))
            Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, gnn.GNN_MEAN, plan=dg.plan_fwd,
                                  flags=layout_flags | hint, max_slices=max_slices)
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dX, el.n, f, gnn.GNN_MEAN, plan=dg.plan_bwd,
                                  flags=layout_flags | hint, max_slices=max_slices)
            torch.cuda.synchronize()
            assert_close(Y, Yo, S, bf16, f"fwd hints={hint}")
            assert_close(dX, dXo, St, bf16, f"bwd hints={hint}")
            outs.append((Y, dX))
        assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("dtype,f", [(torch.float32, 36), (torch.float32, 68), (torch.float32, 100), (torch.float32, 132),
                                     (torch.float32, 237), (torch.bfloat16, 72), (torch.bfloat16, 136), (torch.bfloat16, 200)])
@pytest.mark.parametrize("max_slices", [0, 2, 4])
def test_dense_tail_table(dtype, f, max_slices):
    """Widths whose last line holds at most 64 bytes: the padded copy keeps those columns in a
    table of their own (several rows per L2 line).  Forced on a small graph with hub rows; every
    op in both directions, including the own-row term of SAGE_GCN and the scale folded into the copy."""
    el = synth.rmat_symmetric(5000, 140000, (0.57, 0.19, 0.19, 0.05), 12)
    bf16 = dtype == torch.bfloat16
    dg = device_graph(el, plan_params=gnn.make_plan_params([4, 32, 256], 64))
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    X = synth.normal_features(el.n, f, 5, dtype=dtype)
    Xd = X.to(DEV)
    for op_name in ("sum", "mean", "gcn", "sage"):
        op = OP_CODE[op_name]
        Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
        dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, op, plan=dg.plan_fwd,
                              flags=gnn.GNN_FLAG_FORCE_PADDED_COPY, max_slices=max_slices)
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dX, el.n, f, op, plan=dg.plan_bwd,
                              flags=gnn.GNN_FLAG_FORCE_PADDED_COPY, max_slices=max_slices)
        torch.cuda.synchronize()
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, dout=dout, nthreads=8, want_scale=True)
        dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, din=din, nthreads=8, want_scale=True)
        assert_close(Y, Yo, S, bf16, f"fwd {op_name} F={f} S<={max_slices}")
        assert_close(dX, dXo, St, bf16, f"bwd {op_name} F={f} S<={max_slices}")


@pytest.mark.parametrize("dtype,f", [(torch.float32, 100), (torch.float32, 64), (torch.float32, 7), (torch.bfloat16, 136)])
def test_rank_ordered_copy_does_not_change_results(dtype, f):
    """The plan-owned padded copy stores rows by descending gather count and is gathered through a
    rank-mapped index copy; with and without it (and with the cold flag forced on) the output is
    bit-identical, and it matches the oracle: all ops, both directions, hub rows, own-row term."""
    el = synth.rmat_symmetric(7000, 180000, (0.57, 0.19, 0.19, 0.05), 21)
    bf16 = dtype == torch.bfloat16
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    X = synth.normal_features(el.n, f, 6, dtype=dtype)
    Xd = X.to(DEV)
    base = gnn.GNN_FLAG_FORCE_PADDED_COPY
    for op_name in ("mean", "gcn", "sage"):
        op = OP_CODE[op_name]
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, dout=dout, nthreads=8, want_scale=True)
        dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, din=din, nthreads=8, want_scale=True)
        outs = []
        for extra in (gnn.GNN_FLAG_NO_RANK_ORDER | gnn.GNN_FLAG_NO_COLD_HINTS, 0, gnn.GNN_FLAG_FORCE_COLD_HINTS):
            dg = device_graph(el, plan_params=gnn.make_plan_params([4, 32, 256], 64))
            Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, op, plan=dg.plan_fwd, flags=base | extra, max_slices=4)
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dX, el.n, f, op, plan=dg.plan_bwd, flags=base | extra, max_slices=4)
            torch.cuda.synchronize()
            assert_close(Y, Yo, S, bf16, f"fwd {op_name} flags={extra}")
            assert_close(dX, dXo, St, bf16, f"bwd {op_name} flags={extra}")
            outs.append((Y, dX))
        for Y, dX in outs[1:]:
            assert torch.equal(Y, outs[0][0]) and torch.equal(dX, outs[0][1])


@pytest.mark.parametrize("dtype,f", [(torch.float32, 100), (torch.float32, 96), (torch.float32, 300), (torch.float32, 602),
                                     (torch.bfloat16, 200), (torch.bfloat16, 513)])
@pytest.mark.parametrize("max_slices", [0, 2, 8])
def test_slice_tables_do_not_change_results(dtype, f, max_slices):
    """The padded copy of a sliced launch is stored as one table per 128-byte column slice; with
    the row-major copy instead the output is bit-identical, and both match the oracle: rows of
    up to 19 lines (several launches), a dense tail, hub rows, the own-row term, the folded scale."""
    el = synth.rmat_symmetric(4500, 120000, (0.57, 0.19, 0.19, 0.05), 33)
    bf16 = dtype == torch.bfloat16
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    X = synth.normal_features(el.n, f, 9, dtype=dtype)
    Xd = X.to(DEV)
    base = gnn.GNN_FLAG_FORCE_PADDED_COPY
    for op_name in ("mean", "gcn", "sage"):
        op = OP_CODE[op_name]
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, dout=dout, nthreads=8, want_scale=True)
        dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, din=din, nthreads=8, want_scale=True)
        outs = []
        for extra in (gnn.GNN_FLAG_NO_SLICE_TABLES, 0, gnn.GNN_FLAG_NO_RANK_ORDER):
            dg = device_graph(el, plan_params=gnn.make_plan_params([4, 32, 256], 64))
            Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, op, plan=dg.plan_fwd, flags=base | extra,
                                  max_slices=max_slices)
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dX, el.n, f, op, plan=dg.plan_bwd, flags=base | extra,
                                  max_slices=max_slices)
            torch.cuda.synchronize()
            assert_close(Y, Yo, S, bf16, f"fwd {op_name} flags={extra}")
            assert_close(dX, dXo, St, bf16, f"bwd {op_name} flags={extra}")
            outs.append((Y, dX))
        for Y, dX in outs[1:]:
            assert torch.equal(Y, outs[0][0]) and torch.equal(dX, outs[0][1])


@pytest.mark.parametrize("dtype,f", [(torch.float32, 4), (torch.float32, 24), (torch.float32, 31), (torch.float32, 33),
                                     (torch.float32, 50), (torch.float32, 257), (torch.bfloat16, 33), (torch.bfloat16, 65),
                                     (torch.bfloat16, 100)])
def test_default_layout_rules_on_a_mid_size_graph(dtype, f):
    """80,000 vertices x 40 edges: large enough for the default rules to copy rows that are not whole
    lines, that straddle lines or that carry a factor (power-of-two rows, dense tail, slice tables,
    rank order) without any forcing flag; every op, both directions, against the oracle, next to
    the call that gathers in place (narrower loads and another row-group shape there, so the two
    agree within the tolerance, not bit for bit)."""
    el = synth.rmat_symmetric(80000, 3200000, (0.57, 0.19, 0.19, 0.05), 77)
    bf16 = dtype == torch.bfloat16
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    X = synth.normal_features(el.n, f, 12, dtype=dtype)
    Xd = X.to(DEV)
    dg = device_graph(el)
    for op_name in ("mean", "gcn", "sage"):
        op = OP_CODE[op_name]
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, dout=dout, nthreads=8, want_scale=True)
        dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, din=din, nthreads=8, want_scale=True)
        for flags in (0, gnn.GNN_FLAG_NO_PADDED_COPY):
            Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, op, plan=dg.plan_fwd, flags=flags)
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dX, el.n, f, op, plan=dg.plan_bwd, flags=flags)
            torch.cuda.synchronize()
            assert_close(Y, Yo, S, bf16, f"fwd {op_name} flags={flags}")
            assert_close(dX, dXo, St, bf16, f"bwd {op_name} flags={flags}")


def test_one_plan_serves_a_sequence_of_widths_dtypes_and_ops():
    """The plan-owned copy, index copies and factor streams are re-laid out or reused from call to
    call: a seeded random sequence of widths, storage types, ops, directions and layout switches
    on ONE pair of plans (80,000 vertices x 40 edges, where the default rules copy) must match the
    oracle call by call."""
    el = synth.rmat_symmetric(80000, 3200000, (0.57, 0.19, 0.19, 0.05), 79)
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    dg = device_graph(el)
    rng = np.random.default_rng(5)
    for it in range(16):
        f = int(rng.choice([1, 3, 4, 8, 12, 16, 24, 31, 32, 33, 47, 50, 64, 65, 96, 100, 128, 129, 200, 256, 257, 300]))
        dtype = torch.bfloat16 if rng.random() < 0.4 else torch.float32
        op_name = str(rng.choice(["sum", "mean", "gcn", "sage"]))
        fwd = rng.random() < 0.5
        flags = int(rng.choice([0, 0, 0, gnn.GNN_FLAG_NO_PADDED_COPY, gnn.GNN_FLAG_NO_SLICE_TABLES, gnn.GNN_FLAG_NO_RANK_ORDER,
                                gnn.GNN_FLAG_NO_COLUMN_SLICES]))
        max_slices = int(rng.choice([0, 0, 0, 2, 8]))
        X = synth.normal_features(el.n, f, 100 + it, dtype=dtype)
        Xd = X.to(DEV)
        out = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
        op = OP_CODE[op_name]
        what = f"call {it}: f={f} {dtype} {op_name} {'fwd' if fwd else 'bwd'} flags={flags} S<={max_slices}"
        print(what, flush=True)
        if fwd:
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, out, el.n, f, op, plan=dg.plan_fwd, flags=flags, max_slices=max_slices)
            ref, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, dout=dout, nthreads=8, want_scale=True)
        else:
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, out, el.n, f, op, plan=dg.plan_bwd, flags=flags, max_slices=max_slices)
            ref, S = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, din=din, nthreads=8, want_scale=True)
        torch.cuda.synchronize()
        assert_close(out, ref, S, dtype == torch.bfloat16, what)


def test_line_gather_probe_reads_what_it_is_told_to():
    """The bare gather probe behind the measured ceilings: every thread's output is the sum of the 4 floats it
    owns in each line its lane group was given; ids beyond the table are clamped to its last line."""
    lines = 1000
    table = torch.arange(lines * 32, dtype=torch.float32, device=DEV) % 1024
    per = 16
    ids = torch.randint(0, lines + 50, ((1 << 20) * per,), dtype=torch.int32, device=DEV)   # some beyond the table
    out = torch.full((1 << 23,), float("nan"), device=DEV)
    n = gnn.gnn_calib_gather(table, lines, ids, out)
    torch.cuda.synchronize()
    assert n == (1 << 20) * per
    groups = [0, 1, 7, 12345, (1 << 20) - 1]
    t = table.view(lines, 32).cpu()
    for g in groups:
        mine = ids[g * per:(g + 1) * per].clamp(max=lines - 1).long().cpu()
        for sub in (0, 3, 7):
            want = t[mine][:, sub * 4:sub * 4 + 4].double().sum().item()
            assert abs(out[g * 8 + sub].item() - want) <= 1e-3 * max(1.0, abs(want)), (g, sub)
