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
