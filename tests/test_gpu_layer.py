"""GPU parity of the dense update (gnn_matmul on the matrix cores) and of the GraphSAGE layer
(aggregation + update, forward and gradients) against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth
from helpers import device_graph, host_csr

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
# fp32 products are exact on the matrix cores; the accumulation of K terms in fp32 (in tiles of
# 16, partial planes of >= 1024) and the fp32 aggregation before or after it leave an error of
# at most (1e-5 + K * 2^-24) * S in the worst case and ~sqrt(K) * 2^-24 * S typically, S being the
# sum of the absolute values of all terms; gate at 2e-5 * S.
RTOL_LAYER = 2e-5


def _close(g, ref, S, what, rtol=RTOL_LAYER):
    g = g.detach().cpu().numpy().astype(np.float64)
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.isfinite(g).all(), what
    err = np.abs(g - ref)
    bound = rtol * S
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} out of tolerance; worst at {i}: gpu={g[i]!r} "
                             f"oracle={ref[i]!r} err={err[i]:.3e} bound={bound[i]:.3e}")


@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (128, 128, 16), (130, 127, 17), (300, 47, 100), (1000, 256, 100),
                                   (257, 300, 602), (64, 16, 602), (5, 7, 0)])
@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
def test_matmul_every_layout(m, n, k, ta, tb):
    rng = np.random.default_rng(m * 7 + n * 3 + k)
    A = rng.normal(size=(k, m) if ta else (m, k)).astype(np.float32)
    B = rng.normal(size=(n, k) if tb else (k, n)).astype(np.float32)
    bias = rng.normal(size=n).astype(np.float32)
    for use_bias, relu in ((False, False), (True, True)):
        print(f"matmul m={m} n={n} k={k} ta={ta} tb={tb} bias={use_bias} relu={relu}", flush=True)
        C = torch.full((m, n), float("nan"), device=DEV)
        gnn.gnn_matmul(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), C, ta, tb,
                       torch.from_numpy(bias).to(DEV) if use_bias else None, relu)
        torch.cuda.synchronize()
        ref, S = oracle.matmul(A, B, ta, tb, bias if use_bias else None, relu)
        _close(C, ref, np.maximum(S, 1e-30), "matmul")


def test_matmul_strided_and_misaligned():
    rng = np.random.default_rng(5)
    m, n, k = 200, 90, 75
    for lda, ldb, ldc, off in ((75, 90, 90, 1), (80, 96, 100, 0), (77, 91, 93, 3)):
        bufA = torch.from_numpy(rng.normal(size=m * lda + 8).astype(np.float32)).to(DEV)
        bufB = torch.from_numpy(rng.normal(size=k * ldb + 8).astype(np.float32)).to(DEV)
        bufC = torch.full((m * ldc + 8,), float("nan"), device=DEV)
        A = torch.as_strided(bufA, (m, k), (lda, 1), off)
        B = torch.as_strided(bufB, (k, n), (ldb, 1), off)
        C = torch.as_strided(bufC, (m, n), (ldc, 1), off)
        gnn.gnn_matmul(A, B, C)
        torch.cuda.synchronize()
        ref, S = oracle.matmul(A.cpu().numpy(), B.cpu().numpy())
        _close(C, ref, S, f"strided {lda}/{ldb}/{ldc}+{off}")
        written = torch.zeros_like(bufC, dtype=torch.bool)
        torch.as_strided(written, (m, n), (ldc, 1), off).fill_(True)
        assert torch.isnan(bufC[~written]).all(), "stores outside C"


def test_matmul_long_reduction_is_split_and_deterministic():
    """The weight-gradient shape: few output tiles, a reduction over many rows."""
    rng = np.random.default_rng(6)
    rows, fi, fo = 200_000, 100, 47
    Z = rng.normal(size=(rows, fi)).astype(np.float32)
    G = rng.normal(size=(rows, fo)).astype(np.float32)
    need = gnn.gnn_matmul_workspace_bytes(fi, fo, rows)
    assert need > 0
    ws = torch.empty(need // 4, device=DEV)
    Zd, Gd = torch.from_numpy(Z).to(DEV), torch.from_numpy(G).to(DEV)
    out = []
    for _ in range(2):
        C = torch.full((fi, fo), float("nan"), device=DEV)
        gnn.gnn_matmul(Zd, Gd, C, trans_a=True, workspace=ws)
        torch.cuda.synchronize()
        out.append(C.clone())
    assert torch.equal(out[0], out[1])
    ref = Z.astype(np.float64).T @ G.astype(np.float64)   # the oracle's triple loop would take minutes here;
    S = np.abs(Z.astype(np.float64)).T @ np.abs(G.astype(np.float64))  # it is pinned to this very routine
    _close(out[0], ref, S, "split reduction")
    C = torch.full((fi, fo), float("nan"), device=DEV)
    gnn.gnn_matmul(Zd, Gd, C, trans_a=True)  # no workspace: unsplit, still right
    torch.cuda.synchronize()
    _close(C, ref, S, "unsplit long reduction", rtol=2e-4)


@pytest.mark.parametrize("m,n,k,ta,tb", [(128 * 21 + 5, 256, 40, False, False), (128 * 17, 300, 64, False, True),
                                         (256 * 19 + 1, 47, 100, False, False), (128 * 40, 130, 33, True, True)])
def test_matmul_tall_results_with_the_tile_order_for_the_xcds(m, n, k, ta, tb):
    """Many row tiles and a few column tiles: the column tiles of one row tile get workgroup ids 8 apart
    (same XCD), the last group of 8 row tiles is incomplete."""
    rng = np.random.default_rng(m + n)
    A = rng.normal(size=(k, m) if ta else (m, k)).astype(np.float32)
    B = rng.normal(size=(n, k) if tb else (k, n)).astype(np.float32)
    bias = rng.normal(size=n).astype(np.float32)
    C = torch.full((m, n), float("nan"), device=DEV)
    gnn.gnn_matmul(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), C, ta, tb, torch.from_numpy(bias).to(DEV), True)
    torch.cuda.synchronize()
    A64, B64 = A.astype(np.float64), B.astype(np.float64)   # the oracle's loop is pinned to this routine; see above
    opA, opB = (A64.T if ta else A64), (B64.T if tb else B64)
    ref = np.maximum(opA @ opB + bias, 0.0)
    S = np.abs(opA) @ np.abs(opB) + np.abs(bias)
    _close(C, ref, S, "tall product")


def test_matmul_split_reduction_of_several_tiles():
    """Four output tiles and a long reduction: all tiles of one part run on one XCD, parts on all eight."""
    rng = np.random.default_rng(61)
    rows, fi, fo = 70_000, 200, 140
    Z = rng.normal(size=(rows, fi)).astype(np.float32)
    G = rng.normal(size=(rows, fo)).astype(np.float32)
    ws = torch.empty(gnn.gnn_matmul_workspace_bytes(fi, fo, rows) // 4, device=DEV)
    assert ws.numel() >= 16 * fi * fo
    C = torch.full((fi, fo), float("nan"), device=DEV)
    gnn.gnn_matmul(torch.from_numpy(Z).to(DEV), torch.from_numpy(G).to(DEV), C, trans_a=True, workspace=ws)
    torch.cuda.synchronize()
    ref = Z.astype(np.float64).T @ G.astype(np.float64)
    S = np.abs(Z.astype(np.float64)).T @ np.abs(G.astype(np.float64))
    _close(C, ref, S, "split reduction over several tiles")


# ------------------------------------------------------------------ one layer
def _graph(kind):
    if kind == "multi":
        return synth.small_random_multigraph(900, 7000, 3), None
    if kind == "rmat_hubs":
        return synth.rmat_symmetric(4000, 120000, (0.57, 0.19, 0.19, 0.05), 5), gnn.make_plan_params([2, 8, 32, 128], 64)
    raise KeyError(kind)


def _layer_case(el, params, fi, fo, relu, order, seed, use_bias=True, want_dx=True, flags=0):
    rng = np.random.default_rng(seed)
    n = el.n
    dg = device_graph(el, plan_params=params)
    indptr, indices, *_ = host_csr(el)
    X = rng.normal(size=(n, fi)).astype(np.float32)
    W = (rng.normal(size=(fi, fo)) / np.sqrt(fi)).astype(np.float32)
    b = rng.normal(size=fo).astype(np.float32) if use_bias else None
    dH = rng.normal(size=(n, fo)).astype(np.float32)
    what = f"n={n} E={el.e} {fi}->{fo} relu={relu} order={order} bias={use_bias}"
    print(what, flush=True)
    Xd, Wd, dHd = (torch.from_numpy(a).to(DEV) for a in (X, W, dH))
    bd = None if b is None else torch.from_numpy(b).to(DEV)
    saved = torch.full((gnn.gnn_sage_layer_saved_elems(n, fi, fo, order),), float("nan"), device=DEV)
    H = torch.full((n, fo), float("nan"), device=DEV)
    gnn.gnn_sage_layer_fwd(dg.indptr, dg.indices, Xd, Wd, bd, saved, H, dg.plan_fwd, relu=relu, order=order, flags=flags)
    torch.cuda.synchronize()
    Z, Ho, SH = oracle.sage_layer_fwd(indptr, indices, X, W, b, relu)
    _close(H, Ho, SH, "forward " + what)
    # backward; the stored forward output that decides the rectifier's mask is the oracle's, for both sides
    Hs = Ho.astype(np.float32)
    extra = n * fo + 64 if flags & gnn.GNN_LAYER_NO_GATE_FOLD else 0  # room for the masked gradient
    ws = torch.empty(max(1, gnn.gnn_sage_layer_workspace_bytes(n, fi, fo, relu, order) // 4) + extra, device=DEV)
    dX = torch.full((n, fi), float("nan"), device=DEV) if want_dx else None
    dW = torch.full((fi, fo), float("nan"), device=DEV)
    db = torch.full((fo,), float("nan"), device=DEV)
    gnn.gnn_sage_layer_bwd(dg.indptr_t, dg.indices_t, Xd, Wd, saved, torch.from_numpy(Hs).to(DEV), dHd, dX, dW, db,
                           dg.plan_bwd, ws, relu=relu, order=order, flags=flags)
    torch.cuda.synchronize()
    g = oracle.sage_layer_bwd(indptr, indices, X, W, Hs, dH, relu)
    _close(dW, g["dW"][0], g["dW"][1], "dW " + what)
    _close(db, g["db"][0], g["db"][1], "db " + what)
    if want_dx:
        _close(dX, g["dX"][0], g["dX"][1], "dX " + what)


@pytest.mark.parametrize("kind", ["multi", "rmat_hubs"])
@pytest.mark.parametrize("fi,fo", [(100, 256), (256, 47), (602, 16), (5, 3), (64, 64), (33, 130)])
@pytest.mark.parametrize("relu", [True, False])
def test_layer_forward_and_gradients(kind, fi, fo, relu):
    el, params = _graph(kind)
    _layer_case(el, params, fi, fo, relu, order=0, seed=fi + fo)


@pytest.mark.parametrize("order", [1, 2])
@pytest.mark.parametrize("fi,fo", [(100, 256), (256, 47)])
def test_layer_either_order_gives_the_same_layer(order, fi, fo):
    el, params = _graph("rmat_hubs")
    _layer_case(el, params, fi, fo, True, order=order, seed=9)


@pytest.mark.parametrize("order", [0, 1, 2])
@pytest.mark.parametrize("fi,fo", [(100, 256), (256, 47), (64, 64), (40, 132), (130, 33)])
@pytest.mark.parametrize("flags", [gnn.GNN_LAYER_FORCE_PRODUCER_LAYOUT, gnn.GNN_LAYER_NO_PRODUCER_LAYOUT])
def test_layer_producer_side_layouts(order, fi, fo, flags):
    """The matrix a layer's aggregation gathers (X W, the masked output gradient, its product with W^T)
    written by its producer straight into the tables of the plan -- forced here on a small graph, with
    hub rows, a dense tail (47, 100, 130) and both orders -- and, for comparison, never."""
    el, params = _graph("rmat_hubs")
    _layer_case(el, params, fi, fo, True, order=order, seed=21, flags=flags)
    _layer_case(el, params, fi, fo, False, order=order, seed=22, flags=flags, use_bias=False)


@pytest.mark.parametrize("fi,fo", [(100, 256), (40, 47), (64, 64), (20, 24), (130, 133)])
@pytest.mark.parametrize("flags", [0, gnn.GNN_LAYER_NO_GATE_FOLD, gnn.GNN_LAYER_FORCE_PRODUCER_LAYOUT])
def test_layer_backward_with_the_rectifier_folded_into_the_products(fi, fo, flags):
    """Aggregating first, the two backward products read dH and H themselves (the gate is applied while
    the operand is staged, the bias gradient is added up from the staged tiles) -- all three tile shapes of
    the product (outputs of up to 32, up to 64 and more columns), with and without a rectifier, with and
    without an input gradient -- and, for comparison, with the masked gradient written first."""
    el, params = _graph("rmat_hubs")
    _layer_case(el, params, fi, fo, True, order=1, seed=31, flags=flags)
    _layer_case(el, params, fi, fo, False, order=1, seed=32, flags=flags)
    _layer_case(el, params, fi, fo, True, order=1, seed=33, flags=flags, want_dx=False)
    _layer_case(el, params, fi, fo, True, order=1, seed=34, flags=flags, use_bias=False)


@pytest.mark.parametrize("flags", [0, gnn.GNN_LAYER_NO_GATE_FOLD])
def test_layer_backward_folded_rectifier_with_a_split_reduction(flags):
    """Enough vertices that the weight-gradient product splits its reduction: the bias gradient then comes
    in one plane per part and is added in plane order; twice the same bits."""
    el = synth.small_random_multigraph(9500, 60000, 8)
    assert gnn.gnn_matmul_workspace_bytes(72, 40, el.n) > 0
    _layer_case(el, None, 72, 40, True, order=1, seed=41, flags=flags)
    _layer_case(el, None, 24, 140, True, order=0, seed=42, flags=flags)
    big = synth.small_random_multigraph(40000, 150000, 9)   # 39 parts of 4 tiles: the tile order for the XCDs
    _layer_case(big, None, 130, 140, True, order=1, seed=43, flags=flags)
    n, fi, fo = el.n, 24, 140
    dg = device_graph(el)
    g = torch.Generator(device="cpu").manual_seed(3)
    X, W, H, dH = (torch.randn(s_, generator=g).to(DEV) for s_ in ((n, fi), (fi, fo), (n, fo), (n, fo)))
    saved = torch.randn(n, fi, generator=g).to(DEV)
    ws = torch.empty(gnn.gnn_sage_layer_workspace_bytes(n, fi, fo, True, 0) // 4 + n * fo + 64, device=DEV)
    outs = []
    for _ in range(2):
        dX, dW, db = torch.empty(n, fi, device=DEV), torch.empty(fi, fo, device=DEV), torch.empty(fo, device=DEV)
        gnn.gnn_sage_layer_bwd(dg.indptr_t, dg.indices_t, X, W, saved, H, dH, dX, dW, db, dg.plan_bwd, ws, relu=True, order=0,
                               flags=flags)
        torch.cuda.synchronize()
        outs.append((dX, dW, db))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_layer_without_bias_and_without_input_gradient():
    el, params = _graph("multi")
    _layer_case(el, params, 40, 24, True, order=0, seed=10, use_bias=False, want_dx=False)
    _layer_case(el, params, 24, 40, False, order=0, seed=11, use_bias=False, want_dx=False)


def test_layer_gradients_are_reproducible():
    el, params = _graph("rmat_hubs")
    n, fi, fo = el.n, 100, 47
    dg = device_graph(el, plan_params=params)
    X = torch.randn(n, fi, device=DEV)
    W = torch.randn(fi, fo, device=DEV)
    H = torch.randn(n, fo, device=DEV)
    dH = torch.randn(n, fo, device=DEV)
    ws = torch.empty(gnn.gnn_sage_layer_workspace_bytes(n, fi, fo, True, 0) // 4 + n * fo + 64, device=DEV)
    outs = []
    for _ in range(2):
        dX, dW, db = torch.empty(n, fi, device=DEV), torch.empty(fi, fo, device=DEV), torch.empty(fo, device=DEV)
        gnn.gnn_sage_layer_bwd(dg.indptr_t, dg.indices_t, X, W, None, H, dH, dX, dW, db, dg.plan_bwd, ws)
        torch.cuda.synchronize()
        outs.append((dX, dW, db))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_layer_argument_errors():
    el, params = _graph("multi")
    dg = device_graph(el, plan_params=params)
    n = el.n
    X = torch.randn(n, 8, device=DEV)
    W = torch.randn(8, 4, device=DEV)
    H = torch.empty(n, 4, device=DEV)
    saved = torch.empty(n * 8, device=DEV)
    with pytest.raises(gnn.GnnError):   # no plan
        gnn.gnn_sage_layer_fwd(dg.indptr, dg.indices, X, W, None, saved, H, None)
    with pytest.raises(gnn.GnnError):   # workspace too small
        gnn.gnn_sage_layer_bwd(dg.indptr_t, dg.indices_t, X, W, saved, H, H, torch.empty_like(X), torch.empty_like(W), None,
                               dg.plan_bwd, torch.empty(16, device=DEV))
    with pytest.raises(ValueError):
        gnn.gnn_sage_layer_fwd(dg.indptr, dg.indices, X[:, ::2], W, None, saved, H, dg.plan_fwd)


@pytest.mark.timeout(900)
def test_layer_fullsize_sparse_workload():
    """2,449,029 vertices / 123,718,280 edges, the first layer of the paper's model for this graph
    (100 -> 256, aggregate first) and its last (256 -> 47, transform first), default plans.
    Forward: sampled rows against the oracle on the compacted neighbourhood of the sample.
    Backward: the identities that tie the gradients to the forward map, in fp64 on the whole output:
    <G, H> = <dW, W> + <db, b> = <dX, X> + <db, b> with G = dH where H > 0."""
    el = synth.make_graph("rmat_sparse_stack", device=DEV)
    n = el.n
    dg = gnn.build_device_graph(el.dst, el.src, n)
    dst_h, src_h = synth.to_csr_numpy(el)
    indptr = oracle.csr_indptr(dst_h, n)
    deg = np.diff(indptr)
    rng = np.random.default_rng(4)
    rows = np.unique(np.concatenate([np.argsort(deg)[-16:], rng.choice(n, 1500, replace=False), np.flatnonzero(deg == 0)[:8]]))
    # compacted problem: the sampled rows first (their own vectors are needed), then every neighbour
    nbr = np.concatenate([src_h[indptr[r]:indptr[r + 1]] for r in rows]).astype(np.int64)
    ids = np.concatenate([rows, np.setdiff1d(np.unique(nbr), rows)])
    local = np.full(n, -1, dtype=np.int64)
    local[ids] = np.arange(len(ids))
    sub_ptr = np.zeros(len(ids) + 1, dtype=np.int64)
    sub_ptr[1:len(rows) + 1] = np.cumsum(deg[rows])
    sub_ptr[len(rows) + 1:] = sub_ptr[len(rows)]
    sub_idx = local[nbr].astype(np.int32)
    for fi, fo, relu in ((100, 256, True), (256, 47, False)):
        print(f"[fullsize layer] {fi}->{fo} relu={relu}", flush=True)
        X = synth.normal_features(n, fi, 1, device=DEV)
        W = synth.normal_features(fi, fo, 2, device=DEV) / fi ** 0.5
        b = synth.normal_features(1, fo, 3, device=DEV).reshape(fo)
        dH = synth.normal_features(n, fo, 4, device=DEV)
        saved = torch.empty(gnn.gnn_sage_layer_saved_elems(n, fi, fo), device=DEV)
        H = torch.full((n, fo), float("nan"), device=DEV)
        gnn.gnn_sage_layer_fwd(dg.indptr, dg.indices, X, W, b, saved, H, dg.plan_fwd, relu=relu)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(H).all())
        _, Ho, SH = oracle.sage_layer_fwd(sub_ptr, sub_idx, X[torch.from_numpy(ids).to(DEV)].cpu().numpy(), W.cpu().numpy(),
                                          b.cpu().numpy(), relu)
        k = len(rows)
        _close(H[torch.from_numpy(rows).to(DEV)], Ho[:k], SH[:k], f"fullsize forward {fi}->{fo}")
        ws = torch.empty(gnn.gnn_sage_layer_workspace_bytes(n, fi, fo, relu) // 4, device=DEV)
        dX, dW, db = torch.empty((n, fi), device=DEV), torch.empty((fi, fo), device=DEV), torch.empty(fo, device=DEV)
        gnn.gnn_sage_layer_bwd(dg.indptr_t, dg.indices_t, X, W, saved, H, dH, dX, dW, db, dg.plan_bwd, ws, relu=relu)
        torch.cuda.synchronize()
        G = torch.where(H > 0, dH, torch.zeros_like(dH)) if relu else dH
        lhs = (G.double() * H.double()).sum().item()
        scale = (G.double().abs() * H.double().abs()).sum().item() + (db.double().abs() * b.double().abs()).sum().item()
        via_w = (dW.double() * W.double()).sum().item() + (db.double() * b.double()).sum().item()
        via_x = (dX.double() * X.double()).sum().item() + (db.double() * b.double()).sum().item()
        assert abs(lhs - via_w) <= 2e-6 * scale, (lhs, via_w, scale)
        assert abs(lhs - via_x) <= 2e-6 * scale, (lhs, via_x, scale)
        del X, dH, saved, H, ws, dX, G


@pytest.mark.parametrize("seed", range(12))
def test_layer_randomised(seed):
    rng = np.random.default_rng(700 + seed)
    n = int(rng.integers(2, 3000))
    e = int(rng.integers(1, 25 * n + 1))
    if n < 64 or rng.random() < 0.5:
        el = synth.small_random_multigraph(n, e, seed)
    else:
        e = min(e - e % 2, n * (n - 1) // 4 * 2)
        el = synth.rmat_symmetric(n, max(e, 2), (0.57, 0.19, 0.19, 0.05), seed)
    k = int(rng.integers(0, 5))
    thr = sorted(set(int(t) for t in rng.integers(1, 100, size=k)))
    params = gnn.make_plan_params(thr, int(rng.choice([0, 7, 64, 1024])))
    fi = int(rng.choice([1, 3, 16, 31, 47, 100, 129, 300]))
    fo = int(rng.choice([1, 2, 16, 41, 47, 64, 130, 256]))
    _layer_case(el, params, fi, fo, relu=bool(rng.random() < 0.6), order=int(rng.integers(0, 3)), seed=seed,
                use_bias=bool(rng.random() < 0.7), want_dx=bool(rng.random() < 0.8))


def test_layer_int64_row_pointers():
    el, params = _graph("rmat_hubs")
    rng = np.random.default_rng(43)
    n, fi, fo = el.n, 48, 20
    dg = device_graph(el, indptr64=True, plan_params=params)
    indptr, indices, *_ = host_csr(el)
    X = rng.normal(size=(n, fi)).astype(np.float32)
    W = rng.normal(size=(fi, fo)).astype(np.float32)
    Xd, Wd = torch.from_numpy(X).to(DEV), torch.from_numpy(W).to(DEV)
    saved = torch.empty(gnn.gnn_sage_layer_saved_elems(n, fi, fo), device=DEV)
    H = torch.empty((n, fo), device=DEV)
    gnn.gnn_sage_layer_fwd(dg.indptr, dg.indices, Xd, Wd, None, saved, H, dg.plan_fwd, relu=False)
    torch.cuda.synchronize()
    _, Ho, SH = oracle.sage_layer_fwd(indptr, indices, X, W, None, False)
    _close(H, Ho, SH, "layer forward, int64 row pointers")
