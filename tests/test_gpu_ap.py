"""GPU parity of the general aggregation primitive (operator table of Table 1) and its
gradients against the CPU oracle: exact for max / min (values and winners), within
1e-5 of the magnitude sum for everything summed."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import RTOL_F32, device_graph, host_csr

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
BINOPS = {"add": 0, "sub": 1, "mul": 2, "div": 3, "copylhs": 4, "copyrhs": 5}
REDUCES = {"sum": 0, "max": 1, "min": 2}


def _graph(kind):
    if kind == "multi":       # duplicates and self-loops, light rows
        return synth.small_random_multigraph(700, 9000, 3), None
    if kind == "rmat_hubs":   # power law; tiny hub pieces so that hub rows are cut into many
        el = synth.rmat_symmetric(3000, 90000, (0.57, 0.19, 0.19, 0.05), 5)
        return el, gnn.make_plan_params([2, 8, 32, 128], 48)
    if kind == "star":        # one row with every edge, everything else empty
        n = 5000
        leaves = torch.arange(1, n, dtype=torch.int32)
        return synth.EdgeList(n, leaves, torch.zeros(n - 1, dtype=torch.int32)), gnn.make_plan_params([4, 64], 100)
    raise KeyError(kind)


def _inputs(rng, n, e_rows, d, ewidth, ties):
    if ties:  # few distinct values: many equal extrema, exact sums
        fV = rng.integers(-2, 3, size=(n, d)).astype(np.float32)
        fE = rng.choice(np.array([-2.0, -1.0, 1.0, 2.0], dtype=np.float32), size=(e_rows, ewidth))
    else:
        fV = rng.normal(size=(n, d)).astype(np.float32)
        fE = rng.normal(size=(e_rows, ewidth)).astype(np.float32)
        fE = (np.sign(fE) * (0.25 + np.abs(fE))).astype(np.float32)
        fE[fE == 0] = 0.25
    return fV, fE


def _close(g, ref, S, what):
    g = g.detach().cpu().numpy().astype(np.float64)
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.isfinite(g).all(), what
    err = np.abs(g - ref)
    bound = RTOL_F32 * S
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} out of tolerance; worst at {i}: gpu={g[i]!r} "
                             f"oracle={ref[i]!r} err={err[i]:.3e} bound={bound[i]:.3e}")
    assert not g[S == 0].any(), what


def _check_all(el, params, d, ewidth, use_eid, ties, seed, binops=BINOPS, reduces=REDUCES, use_plan=True, flags=0,
               max_slices=0):
    rng = np.random.default_rng(seed)
    dg = device_graph(el, plan_params=params, want_perm=True, with_plans=use_plan)
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    n, E = el.n, el.e
    e_rows = E + 5
    eid = rng.permutation(e_rows)[:E].astype(np.int64) if use_eid else None
    fV, fE = _inputs(rng, n, e_rows, d, ewidth, ties)
    dO = rng.normal(size=(n, d)).astype(np.float32)
    fV_d, fE_d, dO_d = (torch.from_numpy(a).to(DEV) for a in (fV, fE, dO))
    eid_d = None if eid is None else torch.from_numpy(eid).to(DEV)
    # edge ids of the transposed graph: CSR position, then the caller's row map
    eid_t = dg.perm if eid is None else eid_d[dg.perm]
    for bname, b in binops.items():
        fv_arg = None if bname == "copyrhs" else fV_d
        fe_arg = None if bname == "copylhs" else fE_d
        for rname, r in reduces.items():
            what = f"n={n} E={E} d={d} ewidth={ewidth} eid={use_eid} ties={ties} {bname}/{rname}"
            print(what, flush=True)
            out = torch.full((n, d), float("nan"), device=DEV)
            arg = torch.full((n, d), -7, dtype=torch.int32, device=DEV) if r else None
            gnn.gnn_ap_fwd(dg.indptr, dg.indices, fv_arg, fe_arg, out, arg, n, d, b, r, plan=dg.plan_fwd, edge_ids=eid_d,
                           flags=flags, max_slices=max_slices)
            torch.cuda.synchronize()
            O, aux = oracle.ap_fwd(indptr, indices, None if bname == "copyrhs" else fV, None if bname == "copylhs" else fE,
                                   d, b, r, eid=eid)
            if rname == "sum":
                _close(out, O, aux, "fwd " + what)
            else:
                assert np.array_equal(out.cpu().numpy().astype(np.float64), O), "fwd values " + what
                assert np.array_equal(arg.cpu().numpy().astype(np.int64), aux), "fwd winners " + what
            # gradients
            arg_h = None if rname == "sum" else aux
            (dV, SV), (dE, SE) = oracle.ap_bwd(indptr, indices, None if bname == "copyrhs" else fV,
                                               None if bname == "copylhs" else fE, dO, d, b, r, eid=eid, arg=arg_h,
                                               n_vertex_rows=n, n_edge_rows=e_rows)
            dfV = torch.full((n, d), float("nan"), device=DEV)
            if rname == "sum":
                gnn.gnn_ap_bwd_vertex(dg.indptr_t, dg.indices_t, dO_d, fe_arg, dfV, n, d, b, plan=dg.plan_bwd, edge_ids=eid_t)
            else:
                gnn.gnn_ap_bwd_vertex_arg(dg.indices, arg, dO_d, fe_arg, dfV, n, n, d, b, edge_ids=eid_d)
            torch.cuda.synchronize()
            _close(dfV, dV, SV, "vertex gradient " + what)
            if bname != "copylhs":
                dfE = torch.full((e_rows, ewidth), float("nan"), device=DEV)
                gnn.gnn_ap_bwd_edge(dg.indptr, dg.indices, arg, fv_arg, fe_arg, dO_d, dfE, n, d, b, plan=dg.plan_fwd, edge_ids=eid_d)
                torch.cuda.synchronize()
                g = dfE.cpu().numpy()
                used = np.zeros(e_rows, dtype=bool)
                used[np.arange(E) if eid is None else eid] = True
                assert np.isnan(g[~used]).all(), "edge gradient wrote rows no edge names: " + what
                _close(dfE[torch.from_numpy(used).to(DEV)], dE[used], SE[used], "edge gradient " + what)


@pytest.mark.parametrize("kind", ["multi", "rmat_hubs", "star"])
@pytest.mark.parametrize("d,ewidth", [(1, 1), (5, 5), (5, 1), (32, 32), (32, 1), (100, 100), (100, 1)])
def test_every_operator_pair(kind, d, ewidth):
    el, params = _graph(kind)
    _check_all(el, params, d, ewidth, use_eid=False, ties=False, seed=d * 7 + ewidth)


@pytest.mark.parametrize("kind", ["multi", "rmat_hubs"])
@pytest.mark.parametrize("d,ewidth", [(8, 8), (8, 1), (36, 36)])
def test_equal_values_pick_the_lowest_edge_position(kind, d, ewidth):
    el, params = _graph(kind)
    _check_all(el, params, d, ewidth, use_eid=False, ties=True, seed=11)


@pytest.mark.parametrize("d,ewidth", [(4, 4), (12, 1), (64, 64)])
def test_edge_ids_remap_the_edge_rows(d, ewidth):
    el, params = _graph("rmat_hubs")
    _check_all(el, params, d, ewidth, use_eid=True, ties=False, seed=13)


@pytest.mark.parametrize("d,ewidth", [(100, 1), (64, 1), (256, 1), (600, 1), (100, 100)])
@pytest.mark.parametrize("max_slices", [8, 2])
def test_padded_copy_and_column_slices(d, ewidth, max_slices):
    """The layout of the sum-only hot path (rows copied to an odd line stride, one-line column
    slices over the XCDs), forced on graphs small enough for the whole-output comparison."""
    el, params = _graph("rmat_hubs")
    ops = {"copylhs": 4, "mul": 2, "sub": 1}
    _check_all(el, params, d, ewidth, use_eid=False, ties=False, seed=d + max_slices, binops=ops,
               flags=gnn.GNN_FLAG_FORCE_PADDED_COPY, max_slices=max_slices)
    _check_all(el, params, d, ewidth, use_eid=True, ties=True, seed=d, binops={"copylhs": 4}, reduces={"max": 1},
               flags=gnn.GNN_FLAG_NO_PADDED_COPY, max_slices=max_slices)
    # cold sources flagged in the plan's index copy and fetched with non-temporal loads
    _check_all(el, params, d, ewidth, use_eid=False, ties=True, seed=d + 1, binops={"copylhs": 4, "mul": 2},
               flags=gnn.GNN_FLAG_FORCE_PADDED_COPY | gnn.GNN_FLAG_FORCE_COLD_HINTS, max_slices=max_slices)


def test_without_a_plan():
    el, _ = _graph("multi")
    _check_all(el, None, 16, 16, use_eid=False, ties=False, seed=17, use_plan=False)
    _check_all(el, None, 7, 1, use_eid=True, ties=True, seed=18, use_plan=False)


def test_wide_rows_span_several_column_slabs():
    el = synth.small_random_multigraph(300, 4000, 21)
    _check_all(el, gnn.make_plan_params([4, 16], 8), 520, 520, False, False, 23, binops={"mul": 2, "div": 3}, reduces=REDUCES)
    _check_all(el, gnn.make_plan_params([4, 16], 8), 301, 1, False, False, 24, binops={"add": 0, "copylhs": 4}, reduces=REDUCES)


def test_strided_and_misaligned_operands():
    """Row strides larger than d and bases off the 16-byte grid take the scalar-access kernels."""
    el, params = _graph("rmat_hubs")
    rng = np.random.default_rng(31)
    dg = device_graph(el, plan_params=params, want_perm=True)
    indptr, indices, *_ = host_csr(el)
    n, E, d = el.n, el.e, 12
    for ldv, lde, ldo, off in ((12, 12, 12, 1), (13, 15, 17, 0), (16, 16, 16, 4)):
        bufV = torch.randn(n * ldv + 8, device=DEV)
        bufE = torch.randn(E * lde + 8, device=DEV).abs() + 0.5
        bufO = torch.full((n * ldo + 8,), float("nan"), device=DEV)
        fV = torch.as_strided(bufV, (n, d), (ldv, 1), off)
        fE = torch.as_strided(bufE, (E, d), (lde, 1), off)
        fO = torch.as_strided(bufO, (n, d), (ldo, 1), off)
        for b, r in ((2, 0), (3, 1), (0, 2)):
            bufO.fill_(float("nan"))
            gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, fE, fO, None, n, d, b, r, plan=dg.plan_fwd)
            torch.cuda.synchronize()
            O, aux = oracle.ap_fwd(indptr, indices, fV.cpu().numpy(), fE.cpu().numpy(), d, b, r)
            if r == 0:
                _close(fO, O, aux, f"strided {ldv}/{lde}/{ldo}+{off} sum")
            else:
                assert np.array_equal(fO.cpu().numpy().astype(np.float64), O)
            written = torch.zeros_like(bufO, dtype=torch.bool)
            torch.as_strided(written, (n, d), (ldo, 1), off).fill_(True)
            assert torch.isnan(bufO[~written]).all(), "stores outside the output rows"


def test_argument_errors_on_the_device():
    el, params = _graph("multi")
    dg = device_graph(el, plan_params=params)
    n, d = el.n, 8
    fV = torch.randn(n, d, device=DEV)
    fE = torch.randn(el.e, d, device=DEV)
    fO = torch.empty(n, d, device=DEV)
    arg = torch.empty(n, d, dtype=torch.int32, device=DEV)
    with pytest.raises(gnn.GnnError):   # winners only exist for max / min
        gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, fE, fO, arg, n, d, 0, 0, plan=dg.plan_fwd)
    with pytest.raises(gnn.GnnError):   # a plan of another graph size
        gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, fE, fO, None, n - 1, d, 0, 0, plan=dg.plan_fwd)
    with pytest.raises(gnn.GnnError):   # copylhs has no edge operand to differentiate
        gnn.gnn_ap_bwd_edge(dg.indptr, dg.indices, None, fV, fE, fO, torch.empty_like(fE), n, d, 4, plan=dg.plan_fwd)
    with pytest.raises(TypeError):
        gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV.double(), fE, fO, None, n, d, 0, 0, plan=dg.plan_fwd)


def test_sum_copylhs_equals_the_hot_path():
    """The general kernel and the tuned sum kernel compute the same aggregation."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.02)
    dg = device_graph(el)
    X = synth.normal_features(el.n, 100, 5).to(DEV)
    Y1 = torch.empty_like(X)
    Y2 = torch.empty_like(X)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y1, el.n, 100, gnn.GNN_SUM, plan=dg.plan_fwd)
    gnn.gnn_ap_fwd(dg.indptr, dg.indices, X, None, Y2, None, el.n, 100, gnn.GNN_BIN_COPY_LHS, gnn.GNN_RED_SUM, plan=dg.plan_fwd)
    torch.cuda.synchronize()
    indptr, indices, *_ = host_csr(el)
    O, S = oracle.ap_fwd(indptr, indices, X.cpu().numpy(), None, 100, 4, 0)
    _close(Y2, O, S, "general kernel")
    _close(Y1, O, S, "hot kernel")


# ------------------------------------------------------------------ full size
def _sub_csr(indptr, indices, rows):
    """CSR holding only `rows` of a larger CSR, plus the global edge positions of its edges."""
    lens = (indptr[rows + 1] - indptr[rows]).astype(np.int64)
    sub_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    pos = np.concatenate([np.arange(indptr[r], indptr[r + 1], dtype=np.int64) for r in rows]) if len(rows) else np.zeros(0, np.int64)
    return sub_ptr, indices[pos], pos


@pytest.mark.timeout(900)
def test_fullsize_sparse_workload_sampled_rows():
    """2,449,029 vertices / 123,718,280 edges, d = 100, default plans: sampled rows of the forward
    results (max with winners, weighted sum), of the vertex gradient (transposed graph, edge rows
    through perm) and the edge gradient of the sampled rows' edges against the oracle; the
    winner scatter is checked through what it conserves."""
    name, d = "rmat_sparse_stack", 100
    print(f"[fullsize general primitive] {name} d={d}", flush=True)
    el = synth.make_graph(name, device=DEV)
    n, E = el.n, el.e
    dg = gnn.build_device_graph(el.dst, el.src, n, want_perm=True)
    fV = synth.normal_features(n, d, 1, device=DEV)
    dO = synth.normal_features(n, d, 2, device=DEV)
    w = synth.gcn_sym_edge_weights(el.dst, el.src, n).to(DEV) * 50.0 + 0.25
    fO = torch.full((n, d), float("nan"), device=DEV)
    arg = torch.full((n, d), -7, dtype=torch.int32, device=DEV)

    dst_h, src_h = synth.to_csr_numpy(el)
    indptr = oracle.csr_indptr(dst_h, n)
    deg = np.diff(indptr)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([np.argsort(deg)[-32:], rng.choice(n, 4000, replace=False), np.flatnonzero(deg == 0)[:8]]))
    sub_ptr, sub_idx, pos = _sub_csr(indptr, src_h, rows)
    rows_d = torch.from_numpy(rows).to(DEV)
    fV_h, dO_h, w_h = fV.cpu().numpy(), dO.cpu().numpy(), w.cpu().numpy()

    # forward, max with winners
    gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, None, fO, arg, n, d, gnn.GNN_BIN_COPY_LHS, gnn.GNN_RED_MAX, plan=dg.plan_fwd)
    torch.cuda.synchronize()
    O, won = oracle.ap_fwd(sub_ptr, sub_idx, fV_h, None, d, oracle.BIN_COPY_LHS, oracle.RED_MAX)
    assert np.array_equal(fO[rows_d].cpu().numpy().astype(np.float64), O)
    won_global = np.where(won >= 0, pos[np.maximum(won, 0)], -1)
    assert np.array_equal(arg[rows_d].cpu().numpy().astype(np.int64), won_global)
    # winner scatter: every non-empty (v, j) hands its dO to exactly one vertex
    dfV = torch.empty(n, d, device=DEV)
    gnn.gnn_ap_bwd_vertex_arg(dg.indices, arg, dO, None, dfV, n, n, d, gnn.GNN_BIN_COPY_LHS)
    torch.cuda.synchronize()
    nonempty = torch.from_numpy(deg > 0).to(DEV)
    want = dO[nonempty].double().sum(0)
    scale = dO[nonempty].double().abs().sum(0)
    assert bool(((dfV.double().sum(0) - want).abs() <= 1e-6 * scale).all())
    never_won = torch.ones(n, dtype=torch.bool, device=DEV)
    never_won[dg.indices[arg[arg >= 0].long()].long()] = False
    assert not dfV[never_won].any()

    # forward, sum of scalar-weighted rows; its edge gradient on the sampled rows' edges
    gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, w, fO, None, n, d, gnn.GNN_BIN_MUL, gnn.GNN_RED_SUM, plan=dg.plan_fwd)
    dw = torch.full((E,), float("nan"), device=DEV)
    gnn.gnn_ap_bwd_edge(dg.indptr, dg.indices, None, fV, w, dO, dw, n, d, gnn.GNN_BIN_MUL, plan=dg.plan_fwd)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dw).all())
    O, S = oracle.ap_fwd(sub_ptr, sub_idx, fV_h, w_h, d, oracle.BIN_MUL, oracle.RED_SUM, eid=pos)
    _close(fO[rows_d], O, S, "fullsize mul/sum")
    (_, _), (dE, SE) = oracle.ap_bwd(sub_ptr, sub_idx, fV_h, w_h[pos], dO_h[rows], d, oracle.BIN_MUL, oracle.RED_SUM)
    _close(dw[torch.from_numpy(pos).to(DEV)].reshape(-1, 1), dE, SE, "fullsize edge gradient")

    # vertex gradient of the same: the primitive over the transposed graph, weights through perm
    gnn.gnn_ap_bwd_vertex(dg.indptr_t, dg.indices_t, dO, w, dfV, n, d, gnn.GNN_BIN_MUL, plan=dg.plan_bwd, edge_ids=dg.perm)
    torch.cuda.synchronize()
    indptr_t, indices_t, perm = oracle.transpose(indptr, src_h)
    rows_t = np.unique(np.concatenate([np.argsort(np.diff(indptr_t))[-32:], rng.choice(n, 4000, replace=False)]))
    subt_ptr, subt_idx, pos_t = _sub_csr(indptr_t, indices_t, rows_t)
    dV, SV = oracle.ap_fwd(subt_ptr, subt_idx, dO_h, w_h, d, oracle.BIN_MUL, oracle.RED_SUM, eid=perm[pos_t])
    _close(dfV[torch.from_numpy(rows_t).to(DEV)], dV, SV, "fullsize vertex gradient")


@pytest.mark.parametrize("seed", range(16))
def test_randomised_graphs_widths_and_plans(seed):
    """Seeded random draws over graph shape, width, edge-feature width, edge-id map and plan
    parameters (bin thresholds, hub piece size, or no plan); three operator pairs per draw."""
    rng = np.random.default_rng(500 + seed)
    n = int(rng.integers(1, 3000))
    e = int(rng.integers(0, 30 * n + 1))
    if n < 64 or rng.random() < 0.5:
        el = synth.small_random_multigraph(n, max(e, 1), seed) if e > 0 else synth.EdgeList(
            n, torch.zeros(0, dtype=torch.int32), torch.zeros(0, dtype=torch.int32))
    else:
        e = min(e - e % 2, n * (n - 1) // 4 * 2)
        el = synth.rmat_symmetric(n, max(e, 2), (0.57, 0.19, 0.19, 0.05), seed)
    d = int(rng.choice([1, 2, 3, 4, 7, 8, 20, 33, 64, 100, 130, 260]))
    ewidth = d if rng.random() < 0.5 else 1
    use_plan = rng.random() < 0.8
    params = None
    if use_plan:
        k = int(rng.integers(0, 5))
        thr = sorted(set(int(t) for t in rng.integers(1, 100, size=k)))
        params = gnn.make_plan_params(thr, int(rng.choice([0, 5, 32, 1024])))
    names_b = list(BINOPS)
    names_r = list(REDUCES)
    picks = {(names_b[int(rng.integers(6))], names_r[int(rng.integers(3))]) for _ in range(3)}
    for bname, rname in picks:
        _check_all(el, params, d, ewidth, use_eid=bool(rng.random() < 0.4), ties=bool(rng.random() < 0.3), seed=seed,
                   binops={bname: BINOPS[bname]}, reduces={rname: REDUCES[rname]}, use_plan=use_plan)


def test_int64_row_pointers():
    el, params = _graph("rmat_hubs")
    rng = np.random.default_rng(41)
    dg = device_graph(el, indptr64=True, plan_params=params, want_perm=True)
    assert dg.indptr.dtype == torch.int64
    indptr, indices, *_ = host_csr(el)
    n, E, d = el.n, el.e, 20
    fV, fE = _inputs(rng, n, E, d, 1, False)
    dO = rng.normal(size=(n, d)).astype(np.float32)
    fV_d, fE_d, dO_d = (torch.from_numpy(a).to(DEV) for a in (fV, fE, dO))
    out = torch.empty((n, d), device=DEV)
    arg = torch.empty((n, d), dtype=torch.int32, device=DEV)
    gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV_d, fE_d, out, arg, n, d, 2, 2, plan=dg.plan_fwd)
    torch.cuda.synchronize()
    O, won = oracle.ap_fwd(indptr, indices, fV, fE, d, 2, 2)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), O) and np.array_equal(arg.cpu().numpy().astype(np.int64), won)
    dfE = torch.empty((E, 1), device=DEV)
    gnn.gnn_ap_bwd_edge(dg.indptr, dg.indices, arg, fV_d, fE_d, dO_d, dfE, n, d, 2, plan=dg.plan_fwd)
    dfV = torch.empty((n, d), device=DEV)
    gnn.gnn_ap_bwd_vertex(dg.indptr_t, dg.indices_t, dO_d, fE_d, dfV, n, d, 2, plan=dg.plan_bwd, edge_ids=dg.perm)
    torch.cuda.synchronize()
    (_, _), (dE, SE) = oracle.ap_bwd(indptr, indices, fV, fE, dO, d, 2, 2, arg=won)
    _close(dfE, dE, SE, "edge gradient, int64 row pointers")
    (dV, SV), _ = oracle.ap_bwd(indptr, indices, fV, fE, dO, d, 2, 0)
    _close(dfV, dV, SV, "vertex gradient, int64 row pointers")


@pytest.mark.parametrize("d", [33, 50])
@pytest.mark.parametrize("use_eid", [False, True])
def test_scalar_edge_gradient_of_odd_widths_on_a_mid_size_graph(d, use_eid):
    """Large enough (80,000 vertices x 40 edges) for a width that is not a multiple of four to take
    the staged routes: the forward call computes in plan-owned padded rows and hands the results
    (values and winners) over at the end, the scalar edge gradient reads zero-padded copies; every
    message, sum and max, with and without an edge-id map."""
    el = synth.rmat_symmetric(80000, 3200000, (0.57, 0.19, 0.19, 0.05), 78)
    _check_all(el, None, d, 1, use_eid=use_eid, ties=False, seed=d, reduces={"sum": REDUCES["sum"], "max": REDUCES["max"]})


def test_winner_scatter_spread_between_runs_is_bounded():
    """gnn_ap_bwd_vertex_arg adds with fp32 hardware atomics, so the order of the additions, and with it
    the last bits, may differ from run to run.  What cannot differ by more than rounding: two fp32 sums
    of the same k terms in different orders are at most 2 (k - 1) 2^-24 sum|terms| apart.  Bound the
    spread of five runs by exactly that, element by element, on a graph whose hubs win thousands of rows."""
    el = synth.rmat_symmetric(20000, 600000, (0.57, 0.19, 0.19, 0.05), 5)
    n, d = el.n, 24
    dg = device_graph(el)
    fV = synth.normal_features(n, d, 1).to(DEV)
    dO = synth.normal_features(n, d, 2).to(DEV)
    fO = torch.empty((n, d), device=DEV)
    arg = torch.empty((n, d), dtype=torch.int32, device=DEV)
    gnn.gnn_ap_fwd(dg.indptr, dg.indices, fV, None, fO, arg, n, d, gnn.GNN_BIN_COPY_LHS, gnn.GNN_RED_MAX, plan=dg.plan_fwd)
    runs = []
    for _ in range(5):
        dfV = torch.full((n, d), float("nan"), device=DEV)
        gnn.gnn_ap_bwd_vertex_arg(dg.indices, arg, dO, None, dfV, n, n, d, gnn.GNN_BIN_COPY_LHS)
        torch.cuda.synchronize()
        runs.append(dfV.double().cpu())
    # per element: number of terms and sum of their magnitudes, from the winners (index plumbing in fp64 on the host)
    a = arg.cpu().long()
    won = a >= 0
    src = dg.indices.cpu().long()[a.clamp(min=0)]
    cols = torch.arange(d).expand(n, d)
    flat = (src * d + cols)[won]
    k = torch.zeros(n * d, dtype=torch.float64).index_add_(0, flat, torch.ones(flat.numel(), dtype=torch.float64)).reshape(n, d)
    S = torch.zeros(n * d, dtype=torch.float64).index_add_(0, flat, dO.double().cpu().abs()[won]).reshape(n, d)
    assert int(k.max()) > 1000                      # hubs do win thousands of rows here
    bound = 2.0 * (k - 1).clamp(min=0) * 2.0 ** -24 * S
    spread = torch.stack(runs).max(0).values - torch.stack(runs).min(0).values
    assert bool((spread <= bound).all()), float((spread - bound).max())
    assert bool((spread[k <= 1] == 0).all())        # a single term is exact whatever the order
    print(f"winner scatter: largest spread between five runs {float(spread.max()):.3e} "
          f"({float((spread / S.clamp(min=1e-30)).max()):.2e} of the magnitude sum)")
