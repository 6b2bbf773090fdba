"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- a dense adjacency product, exact invariants, closed forms,
brute-force recounts, and the arithmetic the paper prints.

test_pins_catch_planted_mistakes then shows the pins have teeth: each of a
list of plausible mistakes (dropped term, wrong index, transposed operand ...)
is planted into a COPY of oracle.c, compiled on the CPU, and must make at
least one pin fail.
"""
import os
import tempfile

import numpy as np
import pytest

import oracle
import synth

OPS = (oracle.OP_SUM, oracle.OP_MEAN, oracle.OP_GCN_SYM, oracle.OP_SAGE_GCN)


# ---------------------------------------------------------------- helpers
def csr_from_edges(dst, src, n):
    """Test-local CSR build (searchsorted on the sorted destination array)."""
    dst = np.asarray(dst, dtype=np.int64)
    indptr = np.searchsorted(dst, np.arange(n + 1), side="left").astype(np.int64)
    return indptr, np.asarray(src, dtype=np.int32)


def dense_operator(dst, src, n, op, w=None):
    """The |V| x |V| matrix the aggregation multiplies X by (Section 2.1:
    f_O = A x f_X), with the MEAN / GCN scalings folded in, all in fp64."""
    A = np.zeros((n, n), dtype=np.float64)
    vals = np.ones(len(dst)) if w is None else np.asarray(w, dtype=np.float32).astype(np.float64)
    np.add.at(A, (dst, src), vals)                       # duplicates add up
    cnt = np.zeros((n, n)); np.add.at(cnt, (dst, src), 1.0)
    din = cnt.sum(axis=1)
    dout = cnt.sum(axis=0)
    if op == oracle.OP_MEAN:
        A = A / np.maximum(din, 1.0)[:, None]
    elif op == oracle.OP_GCN_SYM and w is None:
        A = A / np.sqrt(np.maximum(din, 1.0))[:, None] / np.sqrt(np.maximum(dout, 1.0))[None, :]
    elif op == oracle.OP_SAGE_GCN:                       # (A + I) scaled by 1/(din+1): Section 6.1
        A = (A + np.eye(n)) / (din + 1.0)[:, None]
    return A, din.astype(np.int64), dout.astype(np.int64)


def small_graph(n, e, seed):
    el = synth.small_random_multigraph(n, e, seed)
    dst, src = synth.to_csr_numpy(el)
    return dst, src


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


# ------------------------------------------------------------------- pins
def pin_dense_adjacency():
    for seed, (n, e, f) in enumerate([(5, 9, 3), (17, 60, 4), (64, 700, 7), (33, 20, 5), (64, 4000, 2)]):
        dst, src = small_graph(n, e, seed)
        indptr, indices = csr_from_edges(dst, src, n)
        X = rand((n, f), 100 + seed)
        dY = rand((n, f), 200 + seed)
        w_all = np.random.default_rng(300 + seed).uniform(0.1, 2.0, len(dst)).astype(np.float32)
        indptr_t, indices_t, perm = oracle.transpose(indptr, indices)
        for op in OPS:
            for w in (None, w_all):
                A, din, dout = dense_operator(dst, src, n, op, w)
                Y = oracle.aggregate_fwd(indptr, indices, X, op=op, w=w, dout=dout)
                np.testing.assert_allclose(Y, A @ X.astype(np.float64), rtol=1e-12, atol=1e-12)
                wt = None if w is None else w[perm]
                dX = oracle.aggregate_bwd(indptr_t, indices_t, dY, op=op, wt=wt, din=din)
                np.testing.assert_allclose(dX, A.T @ dY.astype(np.float64), rtol=1e-12, atol=1e-12)


def pin_all_ones_invariant():
    for name, scale in (("er_tiny", 1.0), ("rmat_sparse_stack", 0.002), ("rmat_dense_wide", 0.004)):
        el = synth.make_graph(name, scale=scale)
        dst, src = synth.to_csr_numpy(el)
        n = el.n
        indptr, indices = csr_from_edges(dst, src, n)
        ones = np.ones((n, 3), dtype=np.float32)
        din = np.bincount(dst, minlength=n)
        dout = np.bincount(src, minlength=n)
        Y = oracle.aggregate_fwd(indptr, indices, ones, op=oracle.OP_SUM, nthreads=4)
        assert np.array_equal(Y, np.repeat(din[:, None], 3, axis=1).astype(np.float64))
        Ym = oracle.aggregate_fwd(indptr, indices, ones, op=oracle.OP_MEAN)
        assert np.array_equal(Ym[:, 0], (din > 0).astype(np.float64))
        indptr_t, indices_t, _ = oracle.transpose(indptr, indices)
        dX = oracle.aggregate_bwd(indptr_t, indices_t, ones, op=oracle.OP_SUM)
        assert np.array_equal(dX[:, 1], dout.astype(np.float64))


def pin_adjoint_identity():
    el = synth.make_graph("rmat_sparse_stack", scale=0.001, seed=7)
    dst, src = synth.to_csr_numpy(el)
    # make it properly directed: drop a seeded half of the edges
    keep = np.random.default_rng(5).random(len(dst)) < 0.5
    dst, src = dst[keep], src[keep]
    n = el.n
    indptr, indices = csr_from_edges(dst, src, n)
    indptr_t, indices_t, perm = oracle.transpose(indptr, indices)
    din = np.diff(indptr)
    dout = np.diff(indptr_t)
    X = rand((n, 5), 1)
    dY = rand((n, 5), 2)
    w_all = np.random.default_rng(3).uniform(0.1, 2.0, len(dst)).astype(np.float32)
    for op in OPS:
        for w in (None, w_all):
            Y = oracle.aggregate_fwd(indptr, indices, X, op=op, w=w, dout=dout)
            dX = oracle.aggregate_bwd(indptr_t, indices_t, dY, op=op, wt=None if w is None else w[perm], din=din)
            lhs = float(np.sum(Y * dY.astype(np.float64)))
            rhs = float(np.sum(X.astype(np.float64) * dX))
            assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs)), (op, lhs, rhs)


def pin_closed_forms():
    f = 4
    # directed ring u -> u+1: Y[v] = X[v-1]; the backward pass shifts the other way.
    n = 11
    src = np.arange(n); dst = (src + 1) % n
    order = np.argsort(dst, kind="stable"); dst, src = dst[order], src[order]
    indptr, indices = csr_from_edges(dst, src, n)
    X = rand((n, f), 4)
    Y = oracle.aggregate_fwd(indptr, indices, X)
    assert np.array_equal(Y, np.roll(X, 1, axis=0).astype(np.float64))
    indptr_t, indices_t, _ = oracle.transpose(indptr, indices)
    dX = oracle.aggregate_bwd(indptr_t, indices_t, X)
    assert np.array_equal(dX, np.roll(X, -1, axis=0).astype(np.float64))
    # star: leaves 1..n-1 <-> hub 0
    n = 40
    leaves = np.arange(1, n)
    dst = np.concatenate([np.zeros(n - 1, dtype=np.int64), leaves])
    src = np.concatenate([leaves, np.zeros(n - 1, dtype=np.int64)])
    order = np.lexsort((src, dst)); dst, src = dst[order], src[order]
    indptr, indices = csr_from_edges(dst, src, n)
    X = rand((n, f), 5)
    Y = oracle.aggregate_fwd(indptr, indices, X)
    np.testing.assert_allclose(Y[0], X[1:].astype(np.float64).sum(axis=0), rtol=1e-13)
    assert np.array_equal(Y[1:], np.repeat(X[:1].astype(np.float64), n - 1, axis=0))
    Ym = oracle.aggregate_fwd(indptr, indices, X, op=oracle.OP_MEAN)
    np.testing.assert_allclose(Ym[0], X[1:].astype(np.float64).mean(axis=0), rtol=1e-13)
    Ys = oracle.aggregate_fwd(indptr, indices, X, op=oracle.OP_SAGE_GCN)
    np.testing.assert_allclose(Ys[0], X.astype(np.float64).mean(axis=0), rtol=1e-13)          # hub: mean of all n rows
    np.testing.assert_allclose(Ys[1:], (X[1:].astype(np.float64) + X[0].astype(np.float64)) / 2.0, rtol=1e-13)
    # d-regular circulant graph with all-ones features under GCN_SYM: every entry is 1.
    n, offs = 30, (1, 2, 5)
    s = np.repeat(np.arange(n), 2 * len(offs))
    d = np.concatenate([[(u + o) % n, (u - o) % n] for u in range(n) for o in offs]).ravel()
    order = np.lexsort((s, d)); d, s = d[order], s[order]
    indptr, indices = csr_from_edges(d, s, n)
    Yg = oracle.aggregate_fwd(indptr, indices, np.ones((n, f), np.float32), op=oracle.OP_GCN_SYM,
                              dout=np.bincount(s, minlength=n))
    np.testing.assert_allclose(Yg, 1.0, rtol=1e-14)
    # no edges at all: zeros for every op (SAGE_GCN: the vertex's own vector over 1), rows present.
    indptr = np.zeros(8, dtype=np.int64); indices = np.zeros(0, dtype=np.int32)
    X0 = rand((7, f), 6)
    for op in OPS:
        Y0 = oracle.aggregate_fwd(indptr, indices, X0, op=op, dout=np.zeros(7, np.int64))
        assert Y0.shape == (7, f)
        assert np.array_equal(Y0, X0.astype(np.float64)) if op == oracle.OP_SAGE_GCN else not Y0.any()


def pin_relabel_equivariance():
    n, e, f = 50, 400, 3
    dst, src = small_graph(n, e, 9)
    indptr, indices = csr_from_edges(dst, src, n)
    X = rand((n, f), 8)
    pi = np.random.default_rng(10).permutation(n)          # old id -> new id
    d2, s2 = pi[dst], pi[src]
    order = np.lexsort((s2, d2)); d2, s2 = d2[order], s2[order]
    ip2, ix2 = csr_from_edges(d2, s2, n)
    X2 = np.empty_like(X); X2[pi] = X
    for op in OPS:
        Y = oracle.aggregate_fwd(indptr, indices, X, op=op, dout=np.bincount(src, minlength=n))
        Y2 = oracle.aggregate_fwd(ip2, ix2, X2, op=op, dout=np.bincount(s2, minlength=n))
        np.testing.assert_allclose(Y2[pi], Y, rtol=1e-12, atol=1e-12)


def pin_linearity_and_row_subset():
    n, e, f = 40, 300, 6
    dst, src = small_graph(n, e, 11)
    indptr, indices = csr_from_edges(dst, src, n)
    X1, X2 = rand((n, f), 12), rand((n, f), 13)
    # a, b and the inputs are chosen so a*X1+b*X2 is exact in fp32 (small integers)
    X1 = np.round(X1 * 8).astype(np.float32); X2 = np.round(X2 * 8).astype(np.float32)
    Y = oracle.aggregate_fwd(indptr, indices, (2 * X1 - 3 * X2).astype(np.float32), op=oracle.OP_MEAN)
    Ya = oracle.aggregate_fwd(indptr, indices, X1, op=oracle.OP_MEAN)
    Yb = oracle.aggregate_fwd(indptr, indices, X2, op=oracle.OP_MEAN)
    np.testing.assert_allclose(Y, 2 * Ya - 3 * Yb, rtol=1e-12, atol=1e-12)
    rows = np.array([7, 0, 39, 7, 21])
    Ys, S = oracle.aggregate_fwd(indptr, indices, X1, op=oracle.OP_MEAN, rows=rows, want_scale=True)
    assert np.array_equal(Ys, Ya[rows])
    Sfull = oracle.aggregate_fwd(indptr, indices, np.abs(X1), op=oracle.OP_MEAN)
    np.testing.assert_allclose(S, Sfull[rows], rtol=1e-13)


def pin_transpose_bruteforce():
    for seed, (n, e) in enumerate([(6, 14), (64, 900), (200, 150)]):
        dst, src = small_graph(n, e, 20 + seed)
        indptr, indices = csr_from_edges(dst, src, n)
        assert np.array_equal(oracle.csr_indptr(dst, n), indptr)
        indptr_t, indices_t, perm = oracle.transpose(indptr, indices)
        pos = np.arange(len(dst))
        order = np.lexsort((pos, src))                  # by source, ties by CSR position
        assert np.array_equal(perm, pos[order])
        assert np.array_equal(indices_t, dst[order].astype(np.int32))
        assert np.array_equal(indptr_t, np.searchsorted(src[order], np.arange(n + 1)))


def pin_plan_bruteforce():
    el = synth.make_graph("rmat_sparse_stack", scale=0.002)
    dst, _ = synth.to_csr_numpy(el)
    n = el.n
    indptr = np.searchsorted(dst, np.arange(n + 1)).astype(np.int64)
    deg = np.diff(indptr)
    for thr, chunk in (([1, 4, 16, 64, 256], 100), ([8], 7), ([], 50), ([1, 2, 3], 0)):
        bin_offsets, row_perm, chunks = oracle.plan(indptr, thr, chunk)
        k = len(thr)
        assert bin_offsets[0] == 0 and bin_offsets[-1] == n and len(bin_offsets) == k + 2
        assert np.array_equal(np.sort(row_perm), np.arange(n))
        edges = [0] + list(thr) + [np.iinfo(np.int64).max]
        for b in range(k + 1):
            rows = row_perm[bin_offsets[b]:bin_offsets[b + 1]]
            assert np.all(np.diff(rows) > 0)
            assert np.all((deg[rows] >= edges[b]) & (deg[rows] < edges[b + 1]))
        hub_rows = row_perm[bin_offsets[k]:bin_offsets[k + 1]]
        if chunk == 0:
            assert len(chunks) == 0
            continue
        expect = []
        for v in hub_rows:
            for b in range(indptr[v], indptr[v + 1], chunk):
                expect.append((v, b, min(b + chunk, indptr[v + 1])))
        assert np.array_equal(chunks, np.array(expect, dtype=np.int64).reshape(-1, 3))


PINS = [pin_dense_adjacency, pin_all_ones_invariant, pin_adjoint_identity, pin_closed_forms,
        pin_relabel_equivariance, pin_linearity_and_row_subset, pin_transpose_bruteforce,
        pin_plan_bruteforce]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin()


def test_paper_work_unit(golden_paper):
    """Table 8's work figures are vertices x average degree x features; with
    Table 2's edge count the same product is edges x features (+ one self term
    per vertex), which is the unit the bench reports."""
    g = golden_paper
    n = g["products_vertices"]
    for hop in ("hop2", "hop1", "hop0"):
        bops = n * g["products_table8_avg_degree"] * g[f"products_{hop}_feats"] / 1e9
        assert abs(bops - g[f"products_{hop}_bops"]) < 0.005
    total = sum(g[f"products_{h}_bops"] for h in ("hop2", "hop1", "hop0"))
    assert abs(total - g["products_full_batch_bops"]) < 0.011
    assert round(g["reddit_edges"] / g["reddit_vertices"]) == g["reddit_avg_degree"]
    assert abs(g["products_edges"] / g["products_vertices"] - g["products_avg_degree"]) < 0.05
    # Table 8's 51.5 is Table 3's 50.5 plus the vertex's own feature vector.
    assert abs(g["products_table8_avg_degree"] - (g["products_avg_degree"] + 1.0)) < 1e-9
    w = synth.WORKLOADS
    assert (w["rmat_dense_wide"]["n"], w["rmat_dense_wide"]["e"]) == (g["reddit_vertices"], g["reddit_edges"])
    assert (w["rmat_sparse_stack"]["n"], w["rmat_sparse_stack"]["e"]) == (g["products_vertices"], g["products_edges"])
    assert (w["rmat_capacity"]["n"], w["rmat_capacity"]["e"]) == (g["papers_vertices"], g["papers_edges"])
    assert w["rmat_sparse_stack"]["widths"] == (g["products_hop2_feats"], g["products_hop1_feats"], g["products_hop0_feats"])


# Each entry: (name, text in oracle.c, replacement).  Every one is a mistake a
# tired implementer could make; every one must trip at least one pin.
MUTATIONS = [
    ("fwd_drop_last_edge", "for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {\n            int64_t u = indices[e];\n            double c = 1.0;\n            if (w)",
     "for (int64_t e = indptr[v]; e + 1 < indptr[v + 1]; ++e) {\n            int64_t u = indices[e];\n            double c = 1.0;\n            if (w)"),
    ("fwd_gathers_wrong_row", "const float *x = X + u * ldx;", "const float *x = X + v * ldx;"),
    ("fwd_mean_not_divided", "if (op == OP_MEAN && din > 0) {\n            for (int64_t j = 0; j < F; ++j) acc[j] /= (double)din;",
     "if (op == OP_MEAN && din > 0) {\n            for (int64_t j = 0; j < F; ++j) acc[j] /= 1.0;"),
    ("fwd_weight_ignored", "if (w) c = (double)w[e];", "if (w) c = 1.0;"),
    ("fwd_gcn_uses_din_twice", "c = 1.0 / sqrt((double)at_least_one(dout[u]) * (double)at_least_one(din));",
     "c = 1.0 / sqrt((double)at_least_one(din) * (double)at_least_one(din));"),
    ("bwd_mean_divides_by_own_row", "if (op == OP_MEAN) c /= (double)din[v];", "if (op == OP_MEAN) c /= (double)at_least_one(dout);"),
    ("bwd_mean_dropped", "if (op == OP_MEAN) c /= (double)din[v];", ""),
    ("bwd_gcn_wrong_degree", "c = 1.0 / sqrt((double)at_least_one(dout) * (double)at_least_one(din[v]));",
     "c = 1.0 / sqrt((double)at_least_one(dout) * (double)at_least_one(dout));"),
    ("bwd_sign", "const float *g = dY + v * ldy;\n            for (int64_t j = 0; j < F; ++j) {\n                double t = c * (double)g[j];\n                acc[j] += t;",
     "const float *g = dY + v * ldy;\n            for (int64_t j = 0; j < F; ++j) {\n                double t = c * (double)g[j];\n                acc[j] -= t;"),
    ("sage_self_term_dropped", "acc[j] = (acc[j] + (double)self[j]) / (double)(din + 1);", "acc[j] = acc[j] / (double)(din + 1);"),
    ("sage_divides_by_din", "acc[j] = (acc[j] + (double)self[j]) / (double)(din + 1);", "acc[j] = (acc[j] + (double)self[j]) / (double)at_least_one(din);"),
    ("sage_bwd_self_uses_dout", "double t = (double)self[j] / (double)(din[u] + 1);", "double t = (double)self[j] / (double)(dout + 1);"),
    ("sage_bwd_edge_unscaled", "if (op == OP_SAGE_GCN) c /= (double)(din[v] + 1);", ""),
    ("transpose_not_stable", "int64_t pos = cursor[u]++;", "int64_t pos = indptr_t[u + 1] - 1 - (cursor[u]++ - indptr_t[u]);"),
    ("transpose_perm_off", "perm[pos] = e;", "perm[pos] = e - indptr[v];"),
    ("indptr_off_by_one", "indptr[v + 1] += 1;\n    }\n    for (int64_t v = 0; v < N; ++v) indptr[v + 1] += indptr[v];",
     "indptr[v] += 1;\n    }\n    for (int64_t v = 0; v < N; ++v) indptr[v + 1] += indptr[v];"),
    ("plan_threshold_strict", "if (thresholds[i] <= d) b += 1;\n        row_perm", "if (thresholds[i] < d) b += 1;\n        row_perm"),
    ("plan_chunk_end", "int64_t e = b + hub_chunk < indptr[v + 1] ? b + hub_chunk : indptr[v + 1];", "int64_t e = b + hub_chunk;"),
    ("abs_scale_missing_abs", "if (mag) mag[j] += fabs(t);\n            }\n        }\n        if (op == OP_MEAN && din > 0)", "if (mag) mag[j] += t;\n            }\n        }\n        if (op == OP_MEAN && din > 0)"),
]


@pytest.mark.parametrize("mutation", MUTATIONS, ids=lambda m: m[0])
def test_pins_catch_planted_mistakes(mutation):
    name, old, new = mutation
    src_path = os.path.join(os.path.dirname(oracle.__file__), "oracle.c")
    text = open(src_path).read()
    assert text.count(old) == 1, f"mutation {name}: anchor text must occur exactly once"
    with tempfile.TemporaryDirectory() as tmp:
        c_path = os.path.join(tmp, "mutant.c")
        so_path = os.path.join(tmp, f"mutant_{name}.so")
        with open(c_path, "w") as fh:
            fh.write(text.replace(old, new))
        oracle.compile_c(c_path, so_path)
        oracle.use_library(so_path)
        try:
            caught = []
            for pin in PINS:
                try:
                    pin()
                except (AssertionError, ValueError):
                    caught.append(pin.__name__)
            assert caught, f"no pin noticed the planted mistake '{name}'"
        finally:
            oracle.use_library(None)


def test_pins_under_undefined_behaviour_sanitizer():
    """The oracle is rebuilt with -fsanitize=undefined (no recovery: any finding aborts the
    process) and the pins run against that build in a child process."""
    import subprocess
    import sys
    src_path = os.path.join(os.path.dirname(oracle.__file__), "oracle.c")
    with tempfile.TemporaryDirectory() as tmp:
        so_path = os.path.join(tmp, "oracle_ubsan.so")
        subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-fsanitize=undefined",
                               "-fno-sanitize-recover=all", "-o", so_path, src_path, "-lm"])
        code = ("import sys; sys.path.insert(0, %r); sys.path.insert(0, %r); import oracle; oracle.use_library(%r); "
                "import test_oracle_pins as t; [p() for p in t.PINS]; print('pins ok under ubsan')"
                % (os.path.dirname(os.path.dirname(os.path.abspath(__file__))), os.path.dirname(os.path.abspath(__file__)), so_path))
        out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=600)
        assert out.returncode == 0, out.stderr[-2000:]
        assert "pins ok under ubsan" in out.stdout


# ---------------------------------------------------------------- source-blocked layout of the long rows
@pytest.mark.parametrize("params", [dict(min_degree=8, hot_lines=20, block_lines=50, max_piece=6, rest_min_count=2),
                                    dict(min_degree=2, hot_lines=1, block_lines=7, max_piece=3, rest_min_count=1),
                                    dict(min_degree=32, hot_lines=5000, block_lines=10, max_piece=100, rest_min_count=16)])
def test_blocked_layout_invariants(params):
    """The layout is pinned by what it must satisfy, recounted by brute force: the pieces tile the
    edge array, every piece lies in one row and one block, blocks never go backwards, inside a
    (block, row) run the ranks ascend, the edges of the long rows appear exactly once each with the
    CSR position they came from, and the slots of a row are consecutive in block order."""
    el = synth.rmat_symmetric(700, 9000, (0.57, 0.19, 0.19, 0.05), 5)
    dst, src = synth.to_csr_numpy(el)
    indptr = oracle.csr_indptr(dst, el.n)
    thr = [2, 8, 32, 128]
    ranks, epos, pieces, rowbase, rank = oracle.blocked_layout(indptr, src, thr, **params)
    n = el.n
    count = np.bincount(src, minlength=n)
    # rank: a permutation that orders by descending count, ties by id
    inv = np.empty(n, dtype=np.int64); inv[rank] = np.arange(n)
    assert sorted(rank.tolist()) == list(range(n))
    for a, b in zip(inv[:-1], inv[1:]):
        assert count[a] > count[b] or (count[a] == count[b] and a < b)
    deg = np.diff(indptr)
    long_rows = [v for v in range(n) if deg[v] >= params["min_degree"]]
    assert len(long_rows) == rowbase.shape[0] - 1 and len(long_rows) > 0
    # every edge of a long row exactly once, at its CSR position, with the rank of its source
    assert sorted(epos.tolist()) == sorted(e for v in long_rows for e in range(indptr[v], indptr[v + 1]))
    assert np.array_equal(ranks, rank[src[epos]])
    row_of_edge = np.searchsorted(indptr, epos, side="right") - 1
    hot = min(params["hot_lines"], n)
    rest = max(int((count >= params["rest_min_count"]).sum()), hot)

    def block(r):
        if r < hot:
            return 0
        if r >= rest:
            return 10 ** 9
        return 1 + (r - hot) // params["block_lines"]

    # pieces tile [0, E_b) in order; one row, one block each; blocks non-decreasing; capped length
    pos, last_key, slots_seen = 0, (-1, -1), {}
    order_rows = sorted(long_rows, key=lambda v: (sum(t <= deg[v] for t in thr), v))
    for begin, length, slot, h in pieces.tolist():
        assert begin == pos and 0 < length <= params["max_piece"]
        pos += length
        v = order_rows[h]
        assert set(row_of_edge[begin:begin + length].tolist()) == {v}
        blks = {block(int(r)) for r in ranks[begin:begin + length]}
        assert len(blks) == 1
        key = (blks.pop(), h)
        assert key >= last_key                       # block-major, rows ascending inside a block
        seg = ranks[begin:begin + length]
        assert np.all(seg[1:] >= seg[:-1])
        if key == last_key:                          # a run cut by max_piece: only the last piece may be short
            assert prev_length == params["max_piece"] and ranks[begin] >= ranks[begin - 1]
        last_key, prev_length = key, length
        slots_seen.setdefault(h, []).append(slot)
    assert pos == epos.shape[0]
    for h, slots in slots_seen.items():
        assert slots == list(range(rowbase[h], rowbase[h + 1]))
    assert sorted(slots_seen) == list(range(len(long_rows)))
