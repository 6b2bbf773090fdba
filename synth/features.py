"""Seeded dense inputs: vertex features, output gradients, explicit edge weights."""
from __future__ import annotations

import math

import torch

from .rng import hash_counter, stream_key, uniform01


def _chunks(total: int, step: int):
    for s in range(0, total, step):
        yield s, min(step, total - s)


def uniform_features(n: int, f: int, seed: int, device="cpu", dtype=torch.float32,
                     chunk_rows: int | None = None) -> torch.Tensor:
    """[n, f] values uniform in [-1, 1)."""
    key = stream_key(seed, 51)
    out = torch.empty((n, f), dtype=dtype, device=device)
    flat = out.view(-1)
    step = (chunk_rows or max(1, (1 << 24) // max(f, 1))) * f
    for s, c in _chunks(n * f, step):
        ctr = torch.arange(s, s + c, dtype=torch.int64, device=device)
        u = uniform01(hash_counter(key, ctr))
        flat[s:s + c] = (2.0 * u - 1.0).to(dtype)
    return out


def normal_features(n: int, f: int, seed: int, device="cpu", dtype=torch.float32,
                    chunk_rows: int | None = None) -> torch.Tensor:
    """[n, f] values ~ N(0, 1) (Box-Muller on counter-based uniforms), rounded
    to `dtype` (fp32 or bf16)."""
    k1 = stream_key(seed, 61)
    k2 = stream_key(seed, 62)
    out = torch.empty((n, f), dtype=dtype, device=device)
    flat = out.view(-1)
    step = (chunk_rows or max(1, (1 << 24) // max(f, 1))) * f
    for s, c in _chunks(n * f, step):
        ctr = torch.arange(s, s + c, dtype=torch.int64, device=device)
        u1 = uniform01(hash_counter(k1, ctr))
        u2 = uniform01(hash_counter(k2, ctr))
        r = torch.sqrt(-2.0 * torch.log1p(-u1))  # 1-u1 in (0, 1]
        z = r * torch.cos((2.0 * math.pi) * u2)
        flat[s:s + c] = z.to(dtype)
    return out


def gcn_sym_edge_weights(dst: torch.Tensor, src: torch.Tensor, n: int) -> torch.Tensor:
    """Explicit fp32 weights w_uv = 1/sqrt(deg_u * deg_v) for a symmetrised
    edge list (deg = number of incident directed edges in either orientation,
    equal for both on a symmetric graph).  This is input data for the
    edge-weighted workload: both the library and the oracle read this array."""
    deg_in = torch.bincount(dst.to(torch.int64), minlength=n).to(torch.float64)
    deg_out = torch.bincount(src.to(torch.int64), minlength=n).to(torch.float64)
    w = 1.0 / torch.sqrt(deg_out[src.to(torch.int64)] * deg_in[dst.to(torch.int64)])
    return w.to(torch.float32)
