"""Seeded sweep of the source-blocked path over graph shapes, blocking parameters, widths, types, ops and
weight handling: every case is compared with the fp64 oracle.  The pieces read their per-edge streams in
windows of 32 edges with loads that start anywhere, so the cases vary where pieces begin and end."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import OP_CODE, assert_close, device_graph, host_csr

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SLICED = gnn.GNN_FLAG_FORCE_PADDED_COPY


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(300, 20000))
    deg = float(rng.choice([6, 20, 60, 150]))
    e = int(min(n * deg, n * (n - 1) // 4)) // 2 * 2
    skew = [(0.57, 0.19, 0.19, 0.05), (0.45, 0.22, 0.22, 0.11), (0.25, 0.25, 0.25, 0.25)][int(rng.integers(0, 3))]
    thresholds = [[4, 32, 256], [8, 64], [2, 16, 128, 1024]][int(rng.integers(0, 3))]
    blocking = dict(min_degree=int(rng.choice(thresholds[:2])), hot_lines=int(rng.integers(1, 400)),
                    block_lines=int(rng.integers(1, 900)), max_piece=int(rng.choice([1, 3, 8, 31, 32, 33, 64, 96, 200])),
                    rest_min_count=int(rng.choice([0, 1, 2, 3, 8, 16])))
    bf16 = bool(rng.integers(0, 2))
    f = int(rng.choice([33, 40, 64, 65, 72, 100, 129, 200, 256, 300])) if not bf16 else int(rng.choice([65, 72, 100, 129, 200, 264, 513]))
    op_name = ["sum", "mean", "gcn", "sage"][int(rng.integers(0, 4))]
    weights = int(rng.integers(0, 3))  # 0: none, 1: explicit, 2: explicit and bound to the plans
    if weights and op_name == "sage":
        op_name = "sum"
    return n, e, skew, thresholds, blocking, bf16, f, op_name, weights, int(rng.choice([2, 4, 8]))


@pytest.mark.parametrize("seed", range(24))
def test_blocked_path_on_seeded_shapes(seed):
    n, e, skew, thresholds, blocking, bf16, f, op_name, weights, max_slices = _case(seed)
    print(f"[sweep {seed}] n={n} e={e} thresholds={thresholds} blocking={blocking} bf16={bf16} f={f} op={op_name} "
          f"weights={weights} max_slices={max_slices}", flush=True)
    el = synth.rmat_symmetric(n, e, skew, 50 + seed)
    indptr, indices, indptr_t, indices_t, perm = host_csr(el)
    din, dout = np.diff(indptr), np.diff(indptr_t)
    dtype = torch.bfloat16 if bf16 else torch.float32
    X = synth.normal_features(el.n, f, 60 + seed, dtype=dtype)
    Xd = X.to(DEV)
    wts = (synth.uniform_features(el.e, 1, 70 + seed).reshape(-1) + 0.5) if weights else None
    dg = device_graph(el, weights=wts, plan_params=gnn.make_plan_params(thresholds, 64))
    for plan in (dg.plan_fwd, dg.plan_bwd):
        plan.set_blocking(**blocking)
    if weights == 2:
        dg.plan_fwd.bind_edge_weights(dg.edge_w)
        dg.plan_bwd.bind_edge_weights(dg.edge_w_t)
    op = OP_CODE[op_name]
    w = None if wts is None else wts.numpy()
    Yo, S = oracle.aggregate_fwd(indptr, indices, X.float().numpy(), op=op, w=w, dout=dout, nthreads=8, want_scale=True)
    dXo, St = oracle.aggregate_bwd(indptr_t, indices_t, X.float().numpy(), op=op, wt=None if w is None else w[perm], din=din,
                                   nthreads=8, want_scale=True)
    for rep in range(2):
        Y = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
        dX = torch.full((el.n, f), float("nan"), dtype=dtype, device=DEV)
        gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w, Xd, Y, el.n, f, op, plan=dg.plan_fwd, flags=SLICED, max_slices=max_slices)
        gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t, Xd, dX, el.n, f, op, plan=dg.plan_bwd, flags=SLICED,
                              max_slices=max_slices)
        torch.cuda.synchronize()
        assert_close(Y, Yo, S, bf16, f"sweep {seed} fwd")
        assert_close(dX, dXo, St, bf16, f"sweep {seed} bwd")
    if (din >= blocking["min_degree"]).any():
        assert dg.plan_fwd.blocked_sizes()[2] > 0, "the case was meant to run through pieces"
