"""The five benchmark workloads as seeded recipes (shapes only; no datasets).

Each entry names a graph model, its size and the feature widths / dtype / op it
is run with.  `make_graph` returns the canonical EdgeList; `make_features`
draws X (or dY) for a width.  `scale=` shrinks N and E by the same factor (same
mean degree and skew) so CPU-only tests can use the same recipes.
"""
from __future__ import annotations

import torch

from .features import normal_features, uniform_features
from .graphs import EdgeList, erdos_renyi_directed, rmat_directed, rmat_symmetric

WORKLOADS = {
    # Tiny plumbing case.
    "er_tiny": dict(model="er", n=4096, e=65536, seed=0, widths=(64,), op="sum",
                    dist="uniform", dtype="f32", indptr64=False),
    # Dense-degree / wide-feature case (shape of the paper's Reddit row, Table 2).
    "rmat_dense_wide": dict(model="rmat_sym", n=232965, e=114615892, seed=2,
                            probs=(0.57, 0.19, 0.19, 0.05), widths=(602, 256), op="mean",
                            dist="normal", dtype="f32", indptr64=False),
    # Sparse / medium-feature case (shape of the OGBN-Products row, Table 2);
    # widths are the aggregation widths of the 3-layer stack (Table 8).
    "rmat_sparse_stack": dict(model="rmat_sym", n=2449029, e=123718280, seed=3,
                              probs=(0.57, 0.19, 0.19, 0.05), widths=(100, 256, 256), op="mean",
                              dist="normal", dtype="f32", indptr64=False),
    # Narrow-feature, explicit edge weights.
    "rmat_weighted_narrow": dict(model="rmat_sym", n=132534, e=79000000, seed=4,
                                 probs=(0.45, 0.22, 0.22, 0.11), widths=(8, 64), op="sum",
                                 weighted=True, dist="normal", dtype="f32", indptr64=False),
    # Capacity case (shape of the OGBN-Papers row, Table 2): directed, 64-bit row pointers.
    "rmat_capacity": dict(model="rmat_dir", n=111059956, e=1615685872, seed=5,
                          probs=(0.57, 0.19, 0.19, 0.05), widths=(128,), op="sum+mean",
                          dist="normal", dtype="bf16", indptr64=True),
}


def make_graph(name: str, device="cpu", scale: float = 1.0, seed: int | None = None) -> EdgeList:
    w = WORKLOADS[name]
    n = max(16, int(round(w["n"] * scale)))
    e = max(32, int(round(w["e"] * scale)))
    seed = w["seed"] if seed is None else seed
    if w["model"] == "er":
        return erdos_renyi_directed(n, e, seed, device=device)
    if w["model"] == "rmat_sym":
        e -= e % 2
        return rmat_symmetric(n, e, w["probs"], seed, device=device)
    if w["model"] == "rmat_dir":
        return rmat_directed(n, e, w["probs"], seed, device=device, batch=min(e // 2, 1 << 28))
    raise KeyError(w["model"])


def make_features(name: str, n: int, f: int, seed: int, device="cpu") -> torch.Tensor:
    w = WORKLOADS[name]
    dtype = torch.bfloat16 if w["dtype"] == "bf16" else torch.float32
    if w["dist"] == "uniform":
        return uniform_features(n, f, seed, device=device, dtype=dtype)
    return normal_features(n, f, seed, device=device, dtype=dtype)
