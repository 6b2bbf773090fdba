"""Packed copies kept by the caller (gnn_packed_bytes / gnn_pack_rows / gnn_aggregate_packed): the
result is compared with the fp64 oracle like every other path, and bit for bit with the call that
makes the same copy itself."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import OP_CODE, assert_close, device_graph, host_csr

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _graph():
    return synth.rmat_symmetric(4500, 120000, (0.57, 0.19, 0.19, 0.05), 41)


def _packed(dg, X, f, op, backward):
    n = X.shape[0]
    nbytes = gnn.gnn_packed_bytes(n, f, gnn.GNN_BF16 if X.dtype == torch.bfloat16 else gnn.GNN_F32)
    assert nbytes > 0
    buf = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device=DEV)
    if backward:
        gnn.gnn_pack_rows(dg.indptr_t, dg.indices_t, X, buf, n, f, op, True, plan=dg.plan_bwd)
    else:
        gnn.gnn_pack_rows(dg.indptr, dg.indices, X, buf, n, f, op, False, plan=dg.plan_fwd)
    return buf


@pytest.mark.parametrize("dtype,f", [(torch.float32, 100), (torch.float32, 256), (torch.float32, 40), (torch.float32, 33),
                                     (torch.float32, 602), (torch.bfloat16, 200), (torch.bfloat16, 65), (torch.bfloat16, 513)])
def test_packed_aggregation_matches_the_oracle_and_the_copying_call(dtype, f):
    el = _graph()
    bf16 = dtype == torch.bfloat16
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    X = synth.normal_features(el.n, f, 12, dtype=dtype)
    Xd = X.to(DEV)
    dg = device_graph(el)
    for op_name in ("sum", "mean", "gcn", "sage"):
        op = OP_CODE[op_name]
        Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, dout=dout, nthreads=8, want_scale=True)
        dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, din=din, nthreads=8, want_scale=True)
        pf, pb = _packed(dg, Xd, f, op, False), _packed(dg, Xd, f, op, True)
        for rep in range(2):  # the copy is read, never written: a second call gives the same bits
            Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
            gnn.gnn_aggregate_packed(dg.indptr, dg.indices, None, pf, Y, el.n, f, op, False, plan=dg.plan_fwd)
            gnn.gnn_aggregate_packed(dg.indptr_t, dg.indices_t, None, pb, dX, el.n, f, op, True, plan=dg.plan_bwd)
            torch.cuda.synchronize()
            assert_close(Y, Yo, S, bf16, f"packed fwd {op_name} F={f}")
            assert_close(dX, dXo, St, bf16, f"packed bwd {op_name} F={f}")
            Yc, dXc = torch.empty_like(Y), torch.empty_like(dX)
            gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Yc, el.n, f, op, plan=dg.plan_fwd,
                                  flags=gnn.GNN_FLAG_FORCE_PADDED_COPY | gnn.GNN_FLAG_NO_DENSE_TAIL, max_slices=8)
            gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dXc, el.n, f, op, plan=dg.plan_bwd,
                                  flags=gnn.GNN_FLAG_FORCE_PADDED_COPY | gnn.GNN_FLAG_NO_DENSE_TAIL, max_slices=8)
            torch.cuda.synchronize()
            assert torch.equal(Y, Yc), f"fwd {op_name} F={f}: differs from the copying call"
            assert torch.equal(dX, dXc), f"bwd {op_name} F={f}: differs from the copying call"


def test_packed_aggregation_with_edge_weights_and_strided_input():
    el = _graph()
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    weights = synth.uniform_features(el.e, 1, 5).reshape(-1) + 0.5
    w = weights.numpy()
    f, ld = 72, 80
    Xw = synth.normal_features(el.n, ld, 13)
    X = Xw[:, :f]
    dg = device_graph(el, weights=weights)
    Xd = Xw.to(DEV)[:, :f]
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.numpy().copy(), op=oracle.OP_SUM, w=w, nthreads=8, want_scale=True)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.numpy().copy(), op=oracle.OP_SUM, wt=w[perm], nthreads=8, want_scale=True)
    pf, pb = _packed(dg, Xd, f, gnn.GNN_SUM, False), _packed(dg, Xd, f, gnn.GNN_SUM, True)
    Y = torch.full((el.n, f), float("nan"), device=DEV)
    dX = torch.full((el.n, f), float("nan"), device=DEV)
    gnn.gnn_aggregate_packed(dg.indptr, dg.indices, dg.edge_w, pf, Y, el.n, f, gnn.GNN_SUM, False, plan=dg.plan_fwd)
    gnn.gnn_aggregate_packed(dg.indptr_t, dg.indices_t, dg.edge_w_t, pb, dX, el.n, f, gnn.GNN_SUM, True, plan=dg.plan_bwd)
    torch.cuda.synchronize()
    assert_close(Y, Yo, S, False, "packed weighted fwd")
    assert_close(dX, dXo, St, False, "packed weighted bwd")


def test_packed_sizes_and_argument_checks():
    assert gnn.gnn_packed_bytes(1000, 100, gnn.GNN_F32) == 1000 * 4 * 128              # four lines, the last one padded
    assert gnn.gnn_packed_bytes(1000, 256, gnn.GNN_F32) == 1000 * 256 * 4
    assert gnn.gnn_packed_bytes(1000, 50, gnn.GNN_F32) == 1000 * 64 * 4
    assert gnn.gnn_packed_bytes(1000, 65, gnn.GNN_BF16) == 1000 * 2 * 128
    assert gnn.gnn_packed_bytes(1000, 32, gnn.GNN_F32) == 0                            # one line: no tables
    assert gnn.gnn_packed_bytes(1000, 257 * 32, gnn.GNN_F32) == 0
    assert gnn.gnn_packed_bytes(0, 100, gnn.GNN_F32) == 0 and gnn.gnn_packed_bytes(10, 100, 7) == 0
    el = _graph()
    dg = device_graph(el)
    f = 100
    X = synth.normal_features(el.n, f, 2).to(DEV)
    Y = torch.empty_like(X)
    small = torch.empty(gnn.gnn_packed_bytes(el.n, f, gnn.GNN_F32) // 4 - 1, device=DEV)
    with pytest.raises(gnn.GnnError):
        gnn.gnn_pack_rows(dg.indptr, dg.indices, X, small, el.n, f, gnn.GNN_SUM, False, plan=dg.plan_fwd)
    with pytest.raises(gnn.GnnError):
        gnn.gnn_aggregate_packed(dg.indptr, dg.indices, None, small, Y, el.n, f, gnn.GNN_SUM, False, plan=dg.plan_fwd)
    ok = torch.empty(gnn.gnn_packed_bytes(el.n, f, gnn.GNN_F32) // 4, device=DEV)
    with pytest.raises(gnn.GnnError):   # the row order is a plan's
        gnn.gnn_pack_rows(dg.indptr, dg.indices, X, ok, el.n, f, gnn.GNN_SUM, False, plan=None)
    one_line = torch.empty(el.n * 32, device=DEV)
    with pytest.raises(gnn.GnnError):   # rows of one line are gathered where they lie
        gnn.gnn_pack_rows(dg.indptr, dg.indices, X[:, :32].contiguous(), one_line, el.n, 32, gnn.GNN_SUM, False, plan=dg.plan_fwd)
    torch.cuda.synchronize()


def test_packed_calls_can_be_captured_into_a_graph():
    """After one eager call (plan-owned index copies are built then) neither gnn_pack_rows nor
    gnn_aggregate_packed allocates, records a memset or synchronises: a step that repacks a changing matrix
    and aggregates from the copy replays bit for bit, with eager work between the replays."""
    el = synth.rmat_symmetric(20000, 600000, (0.57, 0.19, 0.19, 0.05), 3)
    dg = device_graph(el, plan_params=gnn.make_plan_params([4, 32, 256], 128))
    f, op = 100, gnn.GNN_SAGE_GCN
    X = synth.normal_features(el.n, f, 1).to(DEV)
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    pf = torch.empty(gnn.gnn_packed_bytes(el.n, f, gnn.GNN_F32) // 4, device=DEV)
    pb = torch.empty_like(pf)

    def step():
        gnn.gnn_pack_rows(dg.indptr, dg.indices, X, pf, el.n, f, op, False, plan=dg.plan_fwd)
        gnn.gnn_aggregate_packed(dg.indptr, dg.indices, None, pf, Y, el.n, f, op, False, plan=dg.plan_fwd)
        gnn.gnn_pack_rows(dg.indptr_t, dg.indices_t, Y, pb, el.n, f, op, True, plan=dg.plan_bwd)
        gnn.gnn_aggregate_packed(dg.indptr_t, dg.indices_t, None, pb, dX, el.n, f, op, True, plan=dg.plan_bwd)

    step()
    torch.cuda.synchronize()
    want = (Y.clone(), dX.clone())
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
        pf.fill_(float("nan"))
        pb.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, want[0]) and torch.equal(dX, want[1]), f"replay {rep}"
        X.mul_(1.25)
        step()
        torch.cuda.synchronize()
        want = (Y.clone(), dX.clone())


def test_packed_copy_on_a_plan_with_source_blocks():
    """The caller-kept copy has no dense tail table (its size depends on N, F and the type only): on a plan with
    source blocks a short last line is one more table of whole lines, served by the pieces like the others, and
    the call gives the bits of the copying call with the same flags."""
    el = _graph()
    indptr, indices, indptr_t, indices_t, _ = host_csr(el)
    f = 100
    X = synth.normal_features(el.n, f, 14)
    Xd = X.to(DEV)
    dg = device_graph(el, plan_params=gnn.make_plan_params([4, 32, 256], 64))
    for plan in (dg.plan_fwd, dg.plan_bwd):
        plan.set_blocking(min_degree=32, hot_lines=96, block_lines=200, max_piece=24, rest_min_count=3)
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.numpy(), op=oracle.OP_MEAN, nthreads=8, want_scale=True)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.numpy(), op=oracle.OP_MEAN, din=np.diff(indptr), nthreads=8, want_scale=True)
    pf, pb = _packed(dg, Xd, f, gnn.GNN_MEAN, False), _packed(dg, Xd, f, gnn.GNN_MEAN, True)
    assert pf.numel() * 4 == el.n * 4 * 128
    Y, dX, Yc, dXc = (torch.full((el.n, f), float("nan"), device=DEV) for _ in range(4))
    gnn.gnn_aggregate_packed(dg.indptr, dg.indices, None, pf, Y, el.n, f, gnn.GNN_MEAN, False, plan=dg.plan_fwd)
    gnn.gnn_aggregate_packed(dg.indptr_t, dg.indices_t, None, pb, dX, el.n, f, gnn.GNN_MEAN, True, plan=dg.plan_bwd)
    flags = gnn.GNN_FLAG_FORCE_PADDED_COPY | gnn.GNN_FLAG_NO_DENSE_TAIL
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, None, Xd, Yc, el.n, f, gnn.GNN_MEAN, plan=dg.plan_fwd, flags=flags, max_slices=8)
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, None, Xd, dXc, el.n, f, gnn.GNN_MEAN, plan=dg.plan_bwd, flags=flags, max_slices=8)
    torch.cuda.synchronize()
    assert dg.plan_fwd.blocked_sizes()[2] > 0 and dg.plan_bwd.blocked_sizes()[2] > 0
    for what, g, o, s_ in (("packed fwd", Y, Yo, S), ("packed bwd", dX, dXo, St)):
        assert_close(g, o, s_, False, what)
    assert torch.equal(Y, Yc) and torch.equal(dX, dXc)
