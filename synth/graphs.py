"""Seeded synthetic graphs as canonical directed edge lists.

All generators return an EdgeList whose edges are unique, free of self-loops
(unless stated) and sorted by (dst, src) -- the order in which a
destination-indexed CSR stores them.  Everything is integer torch arithmetic on
counter-based random bits, so the same seed gives the same graph on CPU and GPU.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

from .rng import hash_counter, mix64, stream_key


@dataclass
class EdgeList:
    """Directed edges u -> v as parallel int32 tensors, sorted by (dst, src)."""
    n: int
    src: torch.Tensor
    dst: torch.Tensor
    meta: dict = field(default_factory=dict)

    @property
    def e(self) -> int:
        return int(self.src.numel())


def _edge_list_from_keys(keys: torch.Tensor, n: int, meta: dict) -> EdgeList:
    """keys = dst * n + src, sorted ascending and unique."""
    dst = torch.div(keys, n, rounding_mode="floor")
    src = keys - dst * n
    return EdgeList(n=n, src=src.to(torch.int32), dst=dst.to(torch.int32), meta=meta)


def _trim_to(keys: torch.Tensor, target: int, key: int) -> torch.Tensor:
    """Keep exactly `target` of the sorted unique `keys`: those whose hash is
    smallest.  The choice depends on the key set only, not on draw order."""
    if keys.numel() == target:
        return keys
    h = mix64(keys ^ key)
    # kth smallest hash as threshold; 64-bit hashes of distinct keys are
    # distinct for every workload here (checked by the caller's size assert).
    thresh = torch.sort(h).values[target - 1]
    return keys[h <= thresh]


def _collect_unique(draw, target: int, batch: int, key_trim: int, max_rounds: int = 4096) -> torch.Tensor:
    """Draw batches of candidate keys (negative = rejected) until `target`
    distinct ones exist, then trim to exactly `target`."""
    have = None
    start = 0
    for _ in range(max_rounds):
        k = draw(start, batch)
        start += batch
        k = k[k >= 0]
        k = torch.unique(k)
        have = k if have is None else torch.unique(torch.cat([have, k]))
        if have.numel() >= target:
            out = _trim_to(have, target, key_trim)
            assert out.numel() == target, "hash tie while trimming"
            return out
    raise RuntimeError("could not reach the requested number of distinct edges")


def erdos_renyi_directed(n: int, m: int, seed: int, device="cpu") -> EdgeList:
    """G(n, M): exactly m distinct directed edges, no self-loops."""
    assert m <= n * (n - 1)
    ks = stream_key(seed, 11)
    kd = stream_key(seed, 12)
    kt = stream_key(seed, 13)

    def draw(start: int, count: int) -> torch.Tensor:
        c = torch.arange(start, start + count, dtype=torch.int64, device=device)
        # 31 random bits are ample for the vertex counts used with this model.
        s = ((hash_counter(ks, c) >> 33) & 0x7FFFFFFF) % n
        d = ((hash_counter(kd, c) >> 33) & 0x7FFFFFFF) % n
        key = d * n + s
        return torch.where(s == d, torch.full_like(key, -1), key)

    keys = _collect_unique(draw, m, batch=max(1024, int(m * 1.1)), key_trim=kt)
    return _edge_list_from_keys(keys, n, {"model": "erdos_renyi", "seed": seed, "symmetric": False})


def _scramble(x: torch.Tensor, scale: int, seed: int) -> torch.Tensor:
    """A seeded bijection of [0, 2**scale): keeps R-MAT hubs from clustering at
    small vertex ids."""
    mask = (1 << scale) - 1
    half = (scale + 1) // 2
    a1 = (stream_key(seed, 21) | 1) & mask
    b1 = stream_key(seed, 22) & mask
    a2 = (stream_key(seed, 23) | 1) & mask
    b2 = stream_key(seed, 24) & mask
    x = (x * a1 + b1) & mask
    x = x ^ (x >> half)
    x = (x * a2 + b2) & mask
    x = x ^ (x >> half)
    return x


def _rmat_pairs(start: int, count: int, scale: int, probs, seed: int, device) -> tuple:
    """Endpoints (row, col) in [0, 2**scale) of R-MAT draws start..start+count-1."""
    a, b, c, _d = probs
    ta = int(round(a * 65536))
    tb = int(round((a + b) * 65536))
    tc = int(round((a + b + c) * 65536))
    kq = stream_key(seed, 31)
    ctr = torch.arange(start, start + count, dtype=torch.int64, device=device)
    nwords = (scale + 3) // 4
    row = torch.zeros(count, dtype=torch.int64, device=device)
    col = torch.zeros(count, dtype=torch.int64, device=device)
    for j in range(nwords):
        h = hash_counter(kq, ctr * nwords + j)
        for slot in range(4):
            level = j * 4 + slot
            if level >= scale:
                break
            r = (h >> (16 * slot)) & 0xFFFF
            q = (r >= ta).to(torch.int64) + (r >= tb).to(torch.int64) + (r >= tc).to(torch.int64)
            row = (row << 1) | (q >> 1)
            col = (col << 1) | (q & 1)
    return _scramble(row, scale, seed), _scramble(col, scale, seed)


def rmat_directed(n: int, e: int, probs, seed: int, device="cpu", batch: int | None = None) -> EdgeList:
    """Exactly e distinct directed R-MAT edges on n vertices, no self-loops."""
    scale = max(1, math.ceil(math.log2(n)))
    kt = stream_key(seed, 32)

    def draw(start: int, count: int) -> torch.Tensor:
        r, c = _rmat_pairs(start, count, scale, probs, seed, device)
        key = c * n + r  # row = source, col = destination
        bad = (r >= n) | (c >= n) | (r == c)
        return torch.where(bad, torch.full_like(key, -1), key)

    keys = _collect_unique(draw, e, batch=batch or max(1024, e // 2), key_trim=kt)
    return _edge_list_from_keys(keys, n, {"model": "rmat", "probs": tuple(probs), "seed": seed,
                                          "symmetric": False})


def rmat_symmetric(n: int, e: int, probs, seed: int, device="cpu", batch: int | None = None) -> EdgeList:
    """e/2 distinct undirected R-MAT pairs, each stored as two directed edges."""
    assert e % 2 == 0
    pairs = e // 2
    scale = max(1, math.ceil(math.log2(n)))
    kt = stream_key(seed, 33)

    def draw(start: int, count: int) -> torch.Tensor:
        r, c = _rmat_pairs(start, count, scale, probs, seed, device)
        lo = torch.minimum(r, c)
        hi = torch.maximum(r, c)
        key = lo * n + hi
        bad = (hi >= n) | (r == c)
        return torch.where(bad, torch.full_like(key, -1), key)

    und = _collect_unique(draw, pairs, batch=batch or max(1024, pairs // 2), key_trim=kt)
    lo = torch.div(und, n, rounding_mode="floor")
    hi = und - lo * n
    keys = torch.cat([lo * n + hi, hi * n + lo])  # dst * n + src, both directions
    keys = torch.sort(keys).values
    return _edge_list_from_keys(keys, n, {"model": "rmat", "probs": tuple(probs), "seed": seed,
                                          "symmetric": True})


def _unscramble(x: torch.Tensor, scale: int, seed: int) -> torch.Tensor:
    """Inverse of _scramble on [0, 2**scale)."""
    mask = (1 << scale) - 1
    half = (scale + 1) // 2
    a1 = (stream_key(seed, 21) | 1) & mask
    b1 = stream_key(seed, 22) & mask
    a2 = (stream_key(seed, 23) | 1) & mask
    b2 = stream_key(seed, 24) & mask
    inv1 = pow(a1, -1, 1 << scale)
    inv2 = pow(a2, -1, 1 << scale)
    x = x ^ (x >> half)          # 2 * half >= scale: the xor-shift is its own inverse
    x = ((x - b2) * inv2) & mask
    x = x ^ (x >> half)
    x = ((x - b1) * inv1) & mask
    return x


def relabel(el: EdgeList, kind: str, seed: int = 0) -> EdgeList:
    """The same graph with its vertices renamed (and the edge list brought back into (dst, src)
    order): what a vertex reordering does to an aggregation is a property of the input, so the
    orders live here with the generators.
      "degree":      by descending in-degree, equal degrees by old id
      "rmat_prefix": the order of the R-MAT quadrant recursion (vertices sharing the leading bits of
                     their pre-scramble id become neighbours); `seed` is the graph's seed
      "random":      a seeded random permutation"""
    n = el.n
    dev = el.src.device
    ids = torch.arange(n, dtype=torch.int64, device=dev)
    if kind == "degree":
        deg = torch.bincount(el.dst.long(), minlength=n)
        order = torch.sort(-deg, stable=True).indices
    elif kind == "rmat_prefix":
        scale = max(1, math.ceil(math.log2(n)))
        order = torch.sort(_unscramble(ids, scale, seed), stable=True).indices
    elif kind == "random":
        order = torch.sort(mix64(ids ^ stream_key(seed, 81)), stable=True).indices
    else:
        raise KeyError(kind)
    new_id = torch.empty(n, dtype=torch.int64, device=dev)
    new_id[order] = ids
    keys = torch.sort(new_id[el.dst.long()] * n + new_id[el.src.long()]).values
    meta = dict(el.meta)
    meta["relabel"] = kind
    return _edge_list_from_keys(keys, n, meta)


def small_random_multigraph(n: int, e: int, seed: int, allow_dups: bool = True) -> EdgeList:
    """Tiny test graphs that MAY contain duplicate edges and self-loops (the
    aggregation definition is multigraph-safe and the tests exercise that)."""
    ks = stream_key(seed, 41)
    kd = stream_key(seed, 42)
    c = torch.arange(e, dtype=torch.int64)
    s = ((hash_counter(ks, c) >> 33) & 0x7FFFFFFF) % n
    d = ((hash_counter(kd, c) >> 33) & 0x7FFFFFFF) % n
    key = d * n + s
    key = torch.sort(key).values if allow_dups else torch.unique(key)
    return _edge_list_from_keys(key, n, {"model": "multigraph", "seed": seed, "symmetric": False})


def to_csr_numpy(el: EdgeList):
    """(dst, src) int32 numpy arrays of an EdgeList, for host-side consumers."""
    return el.dst.cpu().numpy().astype(np.int32), el.src.cpu().numpy().astype(np.int32)


def regular_random_neighbours(n_rows: int, degree: int, table_rows: int, seed: int, device="cpu"):
    """(indptr int32[n_rows+1], indices int32[n_rows*degree]) of a bipartite-like gather
    pattern: every row has `degree` neighbours drawn uniformly from [0, table_rows).
    Used to measure what a gather achieves when the gathered table has a given size."""
    key = stream_key(seed, 71)
    ctr = torch.arange(n_rows * degree, dtype=torch.int64, device=device)
    idx = ((hash_counter(key, ctr) >> 33) & 0x7FFFFFFF) % table_rows
    indptr = torch.arange(n_rows + 1, dtype=torch.int64, device=device) * degree
    return indptr.to(torch.int32), idx.to(torch.int32)
