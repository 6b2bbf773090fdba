"""Shared helpers of the GPU parity tests: build a device graph from a synth
EdgeList, run the HIP path through the C ABI, run the oracle on the same bits,
and compare under the stated tolerance."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2104_06700_amd as gnn
import synth

# Tolerances of the floating-point comparison.  Every output element must
# satisfy |gpu - oracle| <= RTOL * S with S = sum_e |c_e * x_e| (the magnitude
# sum the oracle accumulates next to the value; S >= |oracle|).  For bf16
# storage the final rounding of the output is relative to the value itself, so
# the bound is RTOL_BF16 * max(S, |oracle|).
RTOL_F32 = 1e-5
RTOL_BF16 = 2e-2
# ... and, on the elements where a relative error is meaningful (no cancellation worth speaking of:
# |oracle| >= S / WELL_CONDITIONED), the plain relative error |gpu - oracle| / |oracle| must meet the
# same figure.
WELL_CONDITIONED = 10.0

OP_CODE = {"sum": gnn.GNN_SUM, "mean": gnn.GNN_MEAN, "gcn": gnn.GNN_GCN_SYM, "sage": gnn.GNN_SAGE_GCN}


def device_graph(el: synth.EdgeList, weights=None, indptr64=False, plan_params=None, want_perm=False, with_plans=True):
    dev = torch.device("cuda:0")
    dst = el.dst.to(dev)
    src = el.src.to(dev)
    w = None if weights is None else weights.to(dev)
    return gnn.build_device_graph(dst, src, el.n, edge_w=w, indptr64=indptr64, plan_params=plan_params,
                                  want_perm=want_perm, with_plans=with_plans)


def host_csr(el: synth.EdgeList):
    """CSR arrays for the oracle, built by the oracle's own routines."""
    dst, src = synth.to_csr_numpy(el)
    indptr = oracle.csr_indptr(dst, el.n)
    indptr_t, indices_t, perm = oracle.transpose(indptr, src)
    return indptr, src, indptr_t, indices_t, perm


def to_f32_numpy(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float32).numpy()


def assert_close(gpu: torch.Tensor, ref: np.ndarray, scale: np.ndarray, bf16: bool, what: str = ""):
    g = to_f32_numpy(gpu).astype(np.float64)
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    if bf16:
        bound = RTOL_BF16 * np.maximum(scale, np.abs(ref))
    else:
        bound = RTOL_F32 * scale
    err = np.abs(g - ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at {i}: "
                             f"gpu={g[i]!r} oracle={ref[i]!r} |err|={err[i]:.3e} bound={bound[i]:.3e}")
    # plain relative error where the sum is well conditioned
    well = (scale > 0) & (np.abs(ref) * WELL_CONDITIONED >= scale)
    if well.any():
        rel = err[well] / np.abs(ref[well])
        rtol = RTOL_BF16 if bf16 else RTOL_F32
        assert rel.max() <= rtol, f"{what}: relative error {rel.max():.3e} on a well-conditioned element exceeds {rtol}"
    # exact zeros where nothing was summed
    assert not g[scale == 0].any(), f"{what}: rows without edges must be exactly zero"


def strict_relative_error(gpu: torch.Tensor, ref: np.ndarray, scale: np.ndarray) -> float:
    """max |g-o|/|o| over the elements with |o| >= 1e-3 S (a looser notion of well-conditioned than
    the gated one in assert_close); reported only."""
    g = to_f32_numpy(gpu).astype(np.float64)
    ok = np.abs(ref) >= 1e-3 * scale
    ok &= scale > 0
    if not ok.any():
        return 0.0
    return float(np.max(np.abs(g - ref)[ok] / np.abs(ref)[ok]))


def run_fwd(dg, X, op, plan="default", weights=True):
    Y = torch.empty_like(X)
    # poison the output so that rows the kernel forgets to write are caught
    Y.fill_(float("nan"))
    gnn.gnn_aggregate_fwd(dg.indptr, dg.indices, dg.edge_w if weights else None, X, Y, dg.n, X.shape[1], op,
                          plan=dg.plan_fwd if plan == "default" else plan)
    torch.cuda.synchronize()
    return Y


def run_bwd(dg, dY, op, plan="default", weights=True):
    dX = torch.empty_like(dY)
    dX.fill_(float("nan"))
    gnn.gnn_aggregate_bwd(dg.indptr_t, dg.indices_t, dg.edge_w_t if weights else None, dY, dX, dg.n, dY.shape[1], op,
                          plan=dg.plan_bwd if plan == "default" else plan)
    torch.cuda.synchronize()
    return dX
