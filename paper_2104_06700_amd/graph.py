"""Convenience holder for one graph on the device: CSR, transposed CSR and the
two degree-binning plans, all produced by library calls."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

from . import binding as B


@dataclass
class DeviceGraph:
    n: int
    e: int
    indptr: torch.Tensor
    indices: torch.Tensor
    edge_w: Optional[torch.Tensor]
    indptr_t: torch.Tensor
    indices_t: torch.Tensor
    edge_w_t: Optional[torch.Tensor]
    perm: Optional[torch.Tensor]
    plan_fwd: Optional[B.Plan]
    plan_bwd: Optional[B.Plan]


def build_device_graph(dst_sorted: torch.Tensor, src: torch.Tensor, n: int, edge_w: Optional[torch.Tensor] = None,
                       indptr64: bool = False, plan_params: Optional[B.GnnPlanParams] = None,
                       want_perm: bool = False, with_plans: bool = True) -> DeviceGraph:
    """dst_sorted/src: int32 device tensors of the edges u->v sorted by (dst, src)."""
    dev = dst_sorted.device
    e = int(dst_sorted.numel())
    ip_dtype = torch.int64 if indptr64 else torch.int32
    indptr = torch.empty(n + 1, dtype=ip_dtype, device=dev)
    B.gnn_csr_from_sorted_coo(dst_sorted, n, indptr)
    indices = src.contiguous()
    indptr_t = torch.empty(n + 1, dtype=ip_dtype, device=dev)
    indices_t = torch.empty(e, dtype=torch.int32, device=dev)
    perm = torch.empty(e, dtype=torch.int64, device=dev) if want_perm else None
    edge_w_t = torch.empty(e, dtype=torch.float32, device=dev) if edge_w is not None else None
    B.gnn_transpose_csr(indptr, indices, edge_w, n, indptr_t, indices_t, perm, edge_w_t)
    plan_fwd = plan_bwd = None
    if with_plans:
        plan_fwd = B.gnn_plan_create(indptr, indices, n, plan_params)
        plan_bwd = B.gnn_plan_create(indptr_t, indices_t, n, plan_params)
    return DeviceGraph(n, e, indptr, indices, edge_w, indptr_t, indices_t, edge_w_t, perm, plan_fwd, plan_bwd)
