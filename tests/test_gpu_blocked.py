"""Source-blocked pieces of the long rows: the layout is compared bit for bit with the oracle's
definition of it, and the aggregation that runs over it with the fp64 oracle, like every other
path (forward, backward, every op, weights, bf16, dense tail, several launches)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import OP_CODE, assert_close, device_graph, host_csr

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
THRESHOLDS = [4, 32, 256]
BLOCKING = dict(min_degree=32, hot_lines=96, block_lines=200, max_piece=24, rest_min_count=3)
SLICED = gnn.GNN_FLAG_FORCE_PADDED_COPY  # with max_slices > 1: slice tables, which the pieces gather from


def _graph():
    return synth.rmat_symmetric(4500, 120000, (0.57, 0.19, 0.19, 0.05), 33)


def _dg(el, weights=None, blocking=BLOCKING):
    dg = device_graph(el, weights=weights, plan_params=gnn.make_plan_params(THRESHOLDS, 64))
    for plan in (dg.plan_fwd, dg.plan_bwd):
        plan.set_blocking(**blocking)
    return dg


@pytest.mark.parametrize("blocking", [BLOCKING, dict(min_degree=4, hot_lines=7, block_lines=33, max_piece=5, rest_min_count=1),
                                      dict(min_degree=256, hot_lines=100000, block_lines=64, max_piece=1000, rest_min_count=16),
                                      dict(min_degree=32, hot_lines=50, block_lines=300, max_piece=40, rest_min_count=40)])
def test_blocked_layout_bit_exact(blocking):
    el = _graph()
    dg = _dg(el, blocking=blocking)
    X = synth.normal_features(el.n, 64, 1).to(DEV)
    Y = torch.empty_like(X)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y, el.n, 64, gnn.GNN_SUM, plan=dg.plan_fwd, flags=SLICED, max_slices=2)
    torch.cuda.synchronize()
    n_rows, n_edges, n_pieces, n_blocks = dg.plan_fwd.blocked_sizes()
    assert n_pieces > 0 and n_rows > 0
    idx, epos, pieces, rowbase, rank = dg.plan_fwd.export_blocked()
    indptr, indices, *_ = host_csr(el)
    o_idx, o_epos, o_pieces, o_rowbase, o_rank = oracle.blocked_layout(indptr, indices, THRESHOLDS, **blocking)
    assert np.array_equal(rank, o_rank)
    assert np.array_equal(rowbase, o_rowbase)
    assert np.array_equal(pieces, o_pieces)
    assert np.array_equal(idx, o_idx) and np.array_equal(epos, o_epos)
    assert n_edges == o_idx.shape[0] and n_rows == o_rowbase.shape[0] - 1


@pytest.mark.parametrize("dtype,f", [(torch.float32, 100), (torch.float32, 64), (torch.float32, 300), (torch.float32, 602),
                                     (torch.bfloat16, 200), (torch.bfloat16, 513)])
@pytest.mark.parametrize("max_slices", [2, 8])
def test_blocked_aggregation_matches_the_oracle(dtype, f, max_slices):
    el = _graph()
    bf16 = dtype == torch.bfloat16
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    X = synth.normal_features(el.n, f, 9, dtype=dtype)
    Xd = X.to(DEV)
    for op_name in ("sum", "mean", "gcn", "sage"):
        op = OP_CODE[op_name]
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, dout=dout, nthreads=8, want_scale=True)
        dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, din=din, nthreads=8, want_scale=True)
        dg = _dg(el)
        for flags in (SLICED, SLICED | gnn.GNN_FLAG_NO_SOURCE_BLOCKS):
            Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, op, plan=dg.plan_fwd, flags=flags, max_slices=max_slices)
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dX, el.n, f, op, plan=dg.plan_bwd, flags=flags, max_slices=max_slices)
            torch.cuda.synchronize()
            assert_close(Y, Yo, S, bf16, f"fwd {op_name} F={f} flags={flags}")
            assert_close(dX, dXo, St, bf16, f"bwd {op_name} F={f} flags={flags}")
        assert dg.plan_fwd.blocked_sizes()[2] > 0 and dg.plan_bwd.blocked_sizes()[2] > 0


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_blocked_aggregation_with_edge_weights(dtype):
    """Explicit weights are read at the CSR position every piece edge came from."""
    el = _graph()
    bf16 = dtype == torch.bfloat16
    weights = synth.uniform_features(el.e, 1, 77).reshape(-1) + 1.5
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    w = weights.numpy()
    f = 136
    X = synth.normal_features(el.n, f, 10, dtype=dtype)
    Xd = X.to(DEV)
    dg = _dg(el, weights=weights)
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=oracle.OP_MEAN, w=w, nthreads=8, want_scale=True)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=oracle.OP_MEAN, wt=w[perm], din=np.diff(indptr),
                                   nthreads=8, want_scale=True)
    Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
    dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, Xd, Y, el.n, f, gnn.GNN_MEAN, plan=dg.plan_fwd, flags=SLICED, max_slices=4)
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t, Xd, dX, el.n, f, gnn.GNN_MEAN, plan=dg.plan_bwd, flags=SLICED, max_slices=4)
    torch.cuda.synchronize()
    assert dg.plan_fwd.blocked_sizes()[2] > 0
    assert_close(Y, Yo, S, bf16, "weighted fwd")
    assert_close(dX, dXo, St, bf16, "weighted bwd")


@pytest.mark.parametrize("hot_lines,block_lines", [(65536, 65536), (65537, 300), (300, 65537), (20000, 30000)])
def test_blocked_aggregation_with_blocks_at_and_beyond_the_16_bit_range(hot_lines, block_lines):
    """The piece kernel reads 16-bit offsets from a block's first rank where every block but the last spans at
    most 65,536 ranks, and the 32-bit ranks otherwise; both must give the oracle's result at the limit."""
    el = synth.rmat_symmetric(150000, 1500000, (0.5, 0.2, 0.2, 0.1), 5)
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    f = 72
    X = synth.normal_features(el.n, f, 21)
    Xd = X.to(DEV)
    dg = _dg(el, blocking=dict(min_degree=32, hot_lines=hot_lines, block_lines=block_lines, max_piece=48, rest_min_count=1))
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.numpy(), op=oracle.OP_SUM, nthreads=8, want_scale=True)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.numpy(), op=oracle.OP_SUM, nthreads=8, want_scale=True)
    Y = torch.full((el.n, f), float("nan"), device=DEV)
    dX = torch.full((el.n, f), float("nan"), device=DEV)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Y, el.n, f, gnn.GNN_SUM, plan=dg.plan_fwd, flags=SLICED, max_slices=4)
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dX, el.n, f, gnn.GNN_SUM, plan=dg.plan_bwd, flags=SLICED, max_slices=4)
    torch.cuda.synchronize()
    assert dg.plan_fwd.blocked_sizes()[3] >= 3
    assert_close(Y, Yo, S, False, "fwd")
    assert_close(dX, dXo, St, False, "bwd")


def test_weights_bound_to_the_plan_are_streamed_in_piece_order():
    """Explicit weights keep a plan that blocks automatically on the path without pieces, unless they are bound
    to it: then the long rows are pieces that read the plan's copy, which gives the bits of the pieces that read
    the caller's array (a plan with blocking asked for explicitly), and the oracle's values before and after
    the weights change and are bound again."""
    el = synth.rmat_symmetric(140000, 6000000, (0.57, 0.19, 0.19, 0.05), 8)
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    weights = synth.uniform_features(el.e, 1, 31).reshape(-1) + 0.25
    w = weights.numpy()
    f = 72
    X = synth.normal_features(el.n, f, 22)
    Xd = X.to(DEV)
    dg = device_graph(el, weights=weights)                       # automatic blocking
    explicit = device_graph(el, weights=weights)
    for plan in (explicit.plan_fwd, explicit.plan_bwd):
        plan.set_blocking(min_degree=256)                        # pieces whatever the weights

    def run(g, scale=1.0):
        Y = torch.full((el.n, f), float("nan"), device=DEV)
        dX = torch.full((el.n, f), float("nan"), device=DEV)
        gnn.gnn_aggregate_fwd(g.indptr, g.indices, g.edge_w, Xd, Y, el.n, f, gnn.GNN_SUM, plan=g.plan_fwd)
        gnn.gnn_aggregate_bwd(g.indptr_t, g.indices_t, g.edge_w_t, Xd, dX, el.n, f, gnn.GNN_SUM, plan=g.plan_bwd)
        torch.cuda.synchronize()
        return Y, dX

    Yo, S = oracle.aggregate_fwd(indptr, indices, X.numpy(), op=oracle.OP_SUM, w=w, nthreads=8, want_scale=True)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.numpy(), op=oracle.OP_SUM, wt=w[perm], nthreads=8, want_scale=True)
    Y0, dX0 = run(dg)                                            # unbound: no pieces
    assert_close(Y0, Yo, S, False, "unbound fwd")
    assert_close(dX0, dXo, St, False, "unbound bwd")
    assert dg.plan_fwd.blocked_sizes()[2] > 0, "the graph is meant to be one that the plan blocks by itself"
    Y2, dX2 = run(explicit)
    assert_close(Y2, Yo, S, False, "explicit blocking fwd")
    assert not torch.equal(Y2, Y0), "pieces add in another order: the two paths should differ in some bit"
    dg.plan_fwd.bind_edge_weights(dg.edge_w)
    dg.plan_bwd.bind_edge_weights(dg.edge_w_t)
    Y1, dX1 = run(dg)
    assert_close(Y1, Yo, S, False, "bound fwd")
    assert_close(dX1, dXo, St, False, "bound bwd")
    assert torch.equal(Y1, Y2) and torch.equal(dX1, dX2), "bound weights: the pieces' results"
    # the weights change: bind again
    dg.edge_w.mul_(-2.0)
    dg.edge_w_t.mul_(-2.0)
    dg.plan_fwd.bind_edge_weights(dg.edge_w)
    dg.plan_bwd.bind_edge_weights(dg.edge_w_t)
    Y3, dX3 = run(dg)
    assert_close(Y3, -2.0 * Yo, 2.0 * S, False, "rebound fwd")
    assert_close(dX3, -2.0 * dXo, 2.0 * St, False, "rebound bwd")
    # another array, or no binding: the path without pieces again
    other = dg.edge_w.clone()
    Y4 = torch.full((el.n, f), float("nan"), device=DEV)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, other, Xd, Y4, el.n, f, gnn.GNN_SUM, plan=dg.plan_fwd)
    dg.plan_fwd.bind_edge_weights(None)
    Y5 = torch.full((el.n, f), float("nan"), device=DEV)
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, Xd, Y5, el.n, f, gnn.GNN_SUM, plan=dg.plan_fwd)
    torch.cuda.synchronize()
    assert torch.equal(Y4, Y5) and torch.equal(Y4, -2.0 * Y0)


def test_blocked_results_are_reproducible_and_parameters_are_checked():
    el = _graph()
    dg = _dg(el)
    X = synth.normal_features(el.n, 100, 3).to(DEV)
    outs = []
    for _ in range(3):
        Y = torch.full_like(X, float("nan"))
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y, el.n, 100, gnn.GNN_MEAN, plan=dg.plan_fwd, flags=SLICED, max_slices=8)
        torch.cuda.synchronize()
        outs.append(Y)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    with pytest.raises(gnn.GnnError):   # the layout is built: its parameters are fixed
        dg.plan_fwd.set_blocking(min_degree=256)
    fresh = device_graph(el, plan_params=gnn.make_plan_params(THRESHOLDS, 64))
    with pytest.raises(gnn.GnnError):   # not a boundary between two bins
        fresh.plan_fwd.set_blocking(min_degree=100)
    with pytest.raises(gnn.GnnError):
        fresh.plan_fwd.set_blocking(min_degree=32, rest_min_count=41)  # not a boundary of the count histogram
    fresh.plan_fwd.set_blocking(min_degree=-1)  # switched off
    Y = torch.full_like(X, float("nan"))
    gnn.gnn_aggregate_fwd(fresh.indptr, fresh.indices, None, X, Y, el.n, 100, gnn.GNN_MEAN, plan=fresh.plan_fwd, flags=SLICED, max_slices=8)
    torch.cuda.synchronize()
    assert fresh.plan_fwd.blocked_sizes() == (0, 0, 0, 0)


def test_blocked_call_with_its_second_stream_can_be_captured_into_a_graph():
    """The short rows run on a library-owned second stream beside the pieces (forked from and joined to the
    caller's stream inside the call): the whole call is still one unit of work on the caller's stream, can be
    captured, and replays bit for bit; switching the overlap off gives the same bits."""
    el = _graph()
    dg = _dg(el)
    f = 100
    X = synth.normal_features(el.n, f, 4).to(DEV)
    Y, dX = torch.empty_like(X), torch.empty_like(X)

    def step(flags=SLICED):
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, X, Y, el.n, f, gnn.GNN_SAGE_GCN, plan=dg.plan_fwd, flags=flags, max_slices=4)
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Y, dX, el.n, f, gnn.GNN_SAGE_GCN, plan=dg.plan_bwd, flags=flags, max_slices=4)

    step()
    torch.cuda.synchronize()
    assert dg.plan_fwd.blocked_sizes()[2] > 0
    want = (Y.clone(), dX.clone())
    step(SLICED | gnn.GNN_FLAG_NO_SHORT_ROW_OVERLAP)
    torch.cuda.synchronize()
    assert torch.equal(Y, want[0]) and torch.equal(dX, want[1])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        Y.fill_(float("nan"))
        dX.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, want[0]) and torch.equal(dX, want[1]), f"replay {rep}"
        X.mul_(0.75)
        step()
        torch.cuda.synchronize()
        want = (Y.clone(), dX.clone())


def test_calls_with_bound_weights_can_be_captured_into_a_graph():
    """Once the weights are bound and one eager call has run, a weighted call allocates nothing and reads the
    plan's copy: captured, it replays bit for bit, also after the weights were changed and bound again (the
    binding refreshes the copy in place, outside the graph)."""
    el = _graph()
    weights = synth.uniform_features(el.e, 1, 9).reshape(-1) + 0.5
    dg = _dg(el, weights=weights)
    dg.plan_fwd.bind_edge_weights(dg.edge_w)
    dg.plan_bwd.bind_edge_weights(dg.edge_w_t)
    f = 100
    X = synth.normal_features(el.n, f, 6).to(DEV)
    Y, dX = torch.empty_like(X), torch.empty_like(X)

    def step():
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, X, Y, el.n, f, gnn.GNN_SUM, plan=dg.plan_fwd, flags=SLICED, max_slices=4)
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t, Y, dX, el.n, f, gnn.GNN_SUM, plan=dg.plan_bwd, flags=SLICED, max_slices=4)

    step()
    torch.cuda.synchronize()
    assert dg.plan_fwd.blocked_sizes()[2] > 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        step()
        torch.cuda.synchronize()
        want = (Y.clone(), dX.clone())
        Y.fill_(float("nan"))
        dX.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, want[0]) and torch.equal(dX, want[1]), f"replay {rep}"
        dg.edge_w.mul_(0.5)
        dg.edge_w_t.mul_(0.5)
        dg.plan_fwd.bind_edge_weights(dg.edge_w)
        dg.plan_bwd.bind_edge_weights(dg.edge_w_t)
        torch.cuda.synchronize()
