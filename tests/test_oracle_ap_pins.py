"""Pins of the general-primitive oracle (oracle/ap_oracle.c) against things other than itself.

Each pin is a plain function; the last test plants mistakes into a COPY of the C file and
requires at least one pin to notice every one of them.
"""
from __future__ import annotations

import os
import tempfile

import numpy as np
import pytest

import oracle
import synth

BINOPS = {"add": oracle.BIN_ADD, "sub": oracle.BIN_SUB, "mul": oracle.BIN_MUL, "div": oracle.BIN_DIV,
          "copylhs": oracle.BIN_COPY_LHS, "copyrhs": oracle.BIN_COPY_RHS}
REDUCES = {"sum": oracle.RED_SUM, "max": oracle.RED_MAX, "min": oracle.RED_MIN}


def small_graph(n, e, seed):
    el = synth.small_random_multigraph(n, e, seed)
    dst, src = synth.to_csr_numpy(el)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(indptr, dst.astype(np.int64) + 1, 1)
    indptr = np.cumsum(indptr)
    return indptr, src.astype(np.int32), dst.astype(np.int64)


def features(rng, n, e_rows, d, ewidth, away_from_zero=True):
    fV = rng.normal(size=(n, d)).astype(np.float32)
    fE = rng.normal(size=(e_rows, ewidth)).astype(np.float32)
    if away_from_zero:  # divisors stay well away from zero
        fE = (np.sign(fE) * (0.5 + np.abs(fE))).astype(np.float32)
        fE[fE == 0] = 0.5
    return fV, fE


def np_message(binop, x, y):
    """Message table by whole-array numpy arithmetic in the dtype of the operands."""
    return {"add": lambda: x + y, "sub": lambda: x - y, "mul": lambda: x * y, "div": lambda: x / y,
            "copylhs": lambda: x + 0 * y, "copyrhs": lambda: y + 0 * x}[binop]()


def np_forward(binop, reduce, indptr, src, dst, fV, fE, eid, dtype):
    """Independent formulation: gather both operands per edge, one array operation for the
    messages, one ufunc.at scatter-reduction by destination."""
    n = indptr.shape[0] - 1
    d = fV.shape[1]
    rows = np.arange(src.shape[0]) if eid is None else eid
    x = fV[src].astype(dtype)
    y = np.broadcast_to(fE[rows].astype(dtype), x.shape)
    m = np_message(binop, x, y)
    if reduce == "sum":
        out = np.zeros((n, d), dtype=dtype)
        np.add.at(out, dst, m)
        return out, m
    init = -np.inf if reduce == "max" else np.inf
    out = np.full((n, d), init, dtype=dtype)
    (np.maximum if reduce == "max" else np.minimum).at(out, dst, m)
    out[np.diff(indptr) == 0] = 0
    return out, m


def pin_message_table_and_scatter():
    rng = np.random.default_rng(5)
    for case, (n, e, d) in enumerate([(1, 0, 3), (7, 20, 1), (23, 150, 5), (40, 300, 4), (12, 9, 2)]):
        indptr, src, dst = small_graph(n, max(e, 1), 100 + case) if e else (np.zeros(n + 1, np.int64), np.zeros(0, np.int32), np.zeros(0, np.int64))
        E = src.shape[0]
        for ewidth in (d, 1):
            for use_eid in (False, True):
                eid = rng.permutation(E + 3)[:E].astype(np.int64) if use_eid else None
                fV, fE = features(rng, n, E + 3, d, ewidth)
                for bname, b in BINOPS.items():
                    for rname, r in REDUCES.items():
                        O, aux = oracle.ap_fwd(indptr, src, fV, fE, d, b, r, eid=eid)
                        if rname == "sum":
                            ref, m = np_forward(bname, rname, indptr, src, dst, fV, fE, eid, np.float64)
                            assert np.allclose(O, ref, rtol=1e-12, atol=1e-12), (case, bname, rname, ewidth, use_eid)
                            mag = np.zeros_like(ref)
                            np.add.at(mag, dst, np.abs(m))
                            assert np.allclose(aux, mag, rtol=1e-12, atol=1e-12)
                        else:
                            ref, m = np_forward(bname, rname, indptr, src, dst, fV, fE, eid, np.float32)
                            assert np.array_equal(O, ref.astype(np.float64)), (case, bname, rname, ewidth, use_eid)
                            # the winner: lowest position in the row whose message equals the extremum
                            for v in range(n):
                                for j in range(d):
                                    row = range(int(indptr[v]), int(indptr[v + 1]))
                                    want = next((p for p in row if m[p, j] == ref[v, j]), -1)
                                    assert aux[v, j] == want, (case, bname, rname, v, j)


def pin_copylhs_sum_is_adjacency_product():
    rng = np.random.default_rng(6)
    indptr, src, dst = small_graph(30, 200, 7)
    fV = rng.normal(size=(30, 4)).astype(np.float32)
    A = np.zeros((30, 30))
    np.add.at(A, (dst, src.astype(np.int64)), 1.0)
    O, _ = oracle.ap_fwd(indptr, src, fV, None, 4, oracle.BIN_COPY_LHS, oracle.RED_SUM)
    assert np.allclose(O, A @ fV.astype(np.float64), rtol=1e-12, atol=1e-12)
    # mul by a scalar edge feature = weighted adjacency product, which the aggregation oracle also computes
    w = rng.uniform(0.5, 2.0, size=src.shape[0]).astype(np.float32)
    Aw = np.zeros((30, 30))
    np.add.at(Aw, (dst, src.astype(np.int64)), w.astype(np.float64))
    O, _ = oracle.ap_fwd(indptr, src, fV, w, 4, oracle.BIN_MUL, oracle.RED_SUM)
    assert np.allclose(O, Aw @ fV.astype(np.float64), rtol=1e-12, atol=1e-12)
    assert np.allclose(O, oracle.aggregate_fwd(indptr, src, fV, op=oracle.OP_SUM, w=w), rtol=1e-12, atol=1e-12)


def pin_closed_forms():
    # star: every leaf points at vertex 0; leaf k carries the value k
    n = 9
    src = np.arange(1, n, dtype=np.int32)
    indptr = np.array([0] + [n - 1] * n, dtype=np.int64)
    fV = np.arange(n, dtype=np.float32).reshape(n, 1) * np.array([[1.0, -1.0]], dtype=np.float32)
    O, arg = oracle.ap_fwd(indptr, src, fV, None, 2, oracle.BIN_COPY_LHS, oracle.RED_MAX)
    assert O[0].tolist() == [n - 1, -1.0] and arg[0].tolist() == [n - 2, 0]
    assert not O[1:].any() and (arg[1:] == -1).all()
    O, arg = oracle.ap_fwd(indptr, src, fV, None, 2, oracle.BIN_COPY_LHS, oracle.RED_MIN)
    assert O[0].tolist() == [1.0, -(n - 1)] and arg[0].tolist() == [0, n - 2]
    # ties: equal values everywhere -> the first edge of the row wins
    ones = np.ones((n, 2), dtype=np.float32)
    for red in (oracle.RED_MAX, oracle.RED_MIN):
        O, arg = oracle.ap_fwd(indptr, src, ones, None, 2, oracle.BIN_COPY_LHS, red)
        assert O[0].tolist() == [1.0, 1.0] and arg[0].tolist() == [0, 0]
    # directed ring u -> u+1 with edge e stored in row e: copyrhs returns the edge features
    n = 6
    indptr = np.arange(n + 1, dtype=np.int64)
    src = ((np.arange(n) - 1) % n).astype(np.int32)
    fE = np.arange(n * 3, dtype=np.float32).reshape(n, 3)
    for red in (oracle.RED_SUM, oracle.RED_MAX, oracle.RED_MIN):
        O, _ = oracle.ap_fwd(indptr, src, None, fE, 3, oracle.BIN_COPY_RHS, red)
        assert np.array_equal(O, fE.astype(np.float64))
    # sub then add of the same edge feature is the identity on a ring; div by 2 halves
    fV = np.linspace(-1, 1, n * 3, dtype=np.float32).reshape(n, 3)
    O, _ = oracle.ap_fwd(indptr, src, fV, np.full((n, 1), 2.0, np.float32), 3, oracle.BIN_DIV, oracle.RED_SUM)
    assert np.allclose(O, fV[src].astype(np.float64) / 2.0, rtol=0, atol=0)
    O, _ = oracle.ap_fwd(indptr, src, fV, np.full((n, 1), 2.0, np.float32), 3, oracle.BIN_SUB, oracle.RED_MIN)
    assert np.array_equal(O, (fV[src] - np.float32(2.0)).astype(np.float64))
    # a negative row under max stays negative (the reduction does not start from zero)
    O, _ = oracle.ap_fwd(indptr, src, -np.abs(fV) - 1, None, 3, oracle.BIN_COPY_LHS, oracle.RED_MAX)
    assert (O < 0).all()


def pin_gradients_by_finite_differences():
    rng = np.random.default_rng(8)
    n, d = 6, 2
    indptr, src, dst = small_graph(n, 14, 9)
    E = src.shape[0]
    h = 1e-6
    for ewidth in (d, 1):
        for use_eid in (False, True):
            eid = rng.permutation(E + 2)[:E].astype(np.int64) if use_eid else None
            fV, fE = features(rng, n, E + 2, d, ewidth)
            dO = rng.normal(size=(n, d)).astype(np.float32)
            for bname, b in BINOPS.items():
                for rname, r in REDUCES.items():
                    def loss(v64, e64):
                        out, _ = np_forward(bname, rname, indptr, src, dst, v64, e64, eid, np.float64)
                        return float((out * dO.astype(np.float64)).sum())
                    arg = None
                    if rname != "sum":
                        _, arg = oracle.ap_fwd(indptr, src, fV, fE, d, b, r, eid=eid)
                    (dV, SV), (dE, SE) = oracle.ap_bwd(indptr, src, fV, fE, dO, d, b, r, eid=eid, arg=arg)
                    v64, e64 = fV.astype(np.float64), fE.astype(np.float64)
                    numV = np.zeros_like(v64)
                    for idx in np.ndindex(*v64.shape):
                        p, m = v64.copy(), v64.copy()
                        p[idx] += h
                        m[idx] -= h
                        numV[idx] = (loss(p, e64) - loss(m, e64)) / (2 * h)
                    numE = np.zeros_like(e64)
                    for idx in np.ndindex(*e64.shape):
                        p, m = e64.copy(), e64.copy()
                        p[idx] += h
                        m[idx] -= h
                        numE[idx] = (loss(v64, p) - loss(v64, m)) / (2 * h)
                    assert np.allclose(dV, numV, rtol=1e-5, atol=1e-7), (bname, rname, ewidth, use_eid, "dV")
                    assert np.allclose(dE, numE, rtol=1e-5, atol=1e-7), (bname, rname, ewidth, use_eid, "dE")
                    assert (SV >= np.abs(dV) - 1e-12).all() and (SE >= np.abs(dE) - 1e-12).all()


def pin_sum_gradients_are_adjoints():
    """mul is bilinear: <dO, O> = <dV, fV> = <dE, fE>; add is linear plus linear: <dO, O> = <dV, fV> + <dE, fE>."""
    rng = np.random.default_rng(10)
    n, d = 50, 6
    indptr, src, dst = small_graph(n, 700, 11)
    E = src.shape[0]
    for ewidth in (d, 1):
        fV, fE = features(rng, n, E, d, ewidth)
        dO = rng.normal(size=(n, d)).astype(np.float32)
        for b, combine in ((oracle.BIN_MUL, lambda a, c: (a, c)), (oracle.BIN_ADD, lambda a, c: (a + c, a + c))):
            O, _ = oracle.ap_fwd(indptr, src, fV, fE, d, b, oracle.RED_SUM)
            (dV, _), (dE, _) = oracle.ap_bwd(indptr, src, fV, fE, dO, d, b, oracle.RED_SUM)
            lhs = float((O * dO).sum())
            a = float((dV * fV).sum())
            c = float((dE * fE).sum())
            want_a, want_c = combine(a, c)
            assert abs(lhs - want_a) <= 1e-9 * (1 + abs(lhs)) and abs(lhs - want_c) <= 1e-9 * (1 + abs(lhs))


PINS = [pin_message_table_and_scatter, pin_copylhs_sum_is_adjacency_product, pin_closed_forms,
        pin_gradients_by_finite_differences, pin_sum_gradients_are_adjoints]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin()


MUTATIONS = [
    ("sub_operands_swapped", "case BIN_SUB: return x - y;", "case BIN_SUB: return y - x;"),
    ("div32_is_mul", "case BIN_DIV: r = x / y; break;", "case BIN_DIV: r = x * y; break;"),
    ("copyrhs_returns_lhs", "default: return y;", "default: return x;"),
    ("edge_ids_ignored_fwd", "int64_t r = eid ? eid[e] : e;\n                float x", "int64_t r = e;\n                float x"),
    ("edge_ids_ignored_bwd", "int64_t r = eid ? eid[e] : e;\n            for", "int64_t r = e;\n            for"),
    ("scalar_edge_feature_reads_column_j", "float y = bin != BIN_COPY_LHS ? fE[r * lde + (ewidth == 1 ? 0 : j)] : 0.0f;",
     "float y = bin != BIN_COPY_LHS ? fE[r * lde + (ewidth == 1 ? 0 : j) * (lde > 1)] : 0.0f; if (ewidth == 1 && j > 0) y = -y;"),
    ("gathers_destination_row", "float x = bin != BIN_COPY_RHS ? fV[u * ldv + j] : 0.0f;", "float x = bin != BIN_COPY_RHS ? fV[v * ldv + j] : 0.0f;"),
    ("last_of_ties_wins", "red == RED_MAX ? m > best : m < best", "red == RED_MAX ? m >= best : m <= best"),
    ("max_min_swapped", "red == RED_MAX ? m > best : m < best", "red == RED_MAX ? m < best : m > best"),
    ("reduction_starts_at_zero", "if (won < 0 || (red == RED_MAX ? m > best : m < best)) {",
     "if (won < 0 ? (red == RED_MAX ? m > 0.0f : m < 0.0f) : (red == RED_MAX ? m > best : m < best)) {"),
    ("empty_row_not_zero", "O[v * d + j] = won >= 0 ? (double)best : 0.0;", "O[v * d + j] = won >= 0 ? (double)best : (red == RED_MAX ? -INFINITY : INFINITY);"),
    ("sub_gradient_sign", "case BIN_SUB: gx = g; gy = -g; break;", "case BIN_SUB: gx = g; gy = g; break;"),
    ("mul_gradients_swapped", "case BIN_MUL: gx = g * y; gy = g * x; break;", "case BIN_MUL: gx = g * x; gy = g * y; break;"),
    ("div_gradient_not_squared", "gy = -g * x / (y * y);", "gy = -g * x / y;"),
    ("div_gradient_lhs", "case BIN_DIV: gx = g / y;", "case BIN_DIV: gx = g * y;"),
    ("copylhs_leaks_into_edges", "case BIN_COPY_LHS: gx = g; gy = 0.0; break;", "case BIN_COPY_LHS: gx = g; gy = g; break;"),
    ("mask_ignored", "if (red != RED_SUM && arg[v * d + j] != e) continue;", ""),
    ("vertex_gradient_lands_on_destination", "dV[u * d + j] += gx;", "dV[v * d + j] += gx;"),
    ("scalar_edge_gradient_keeps_last_column", "dE[k] += gy;", "if (ewidth == 1) dE[k] = gy; else dE[k] += gy;"),
]


@pytest.mark.parametrize("mutation", MUTATIONS, ids=lambda m: m[0])
def test_pins_catch_planted_mistakes(mutation):
    name, old, new = mutation
    src_dir = os.path.dirname(oracle.__file__)
    text = open(os.path.join(src_dir, "ap_oracle.c")).read()
    assert text.count(old) == 1, f"mutation {name}: anchor text must occur exactly once"
    new_text = text.replace(old, new)
    with tempfile.TemporaryDirectory() as tmp:
        c_path = os.path.join(tmp, "mutant_ap.c")
        so_path = os.path.join(tmp, f"mutant_{name}.so")
        with open(c_path, "w") as fh:
            fh.write(new_text)
        oracle.compile_c([os.path.join(src_dir, "oracle.c"), c_path], so_path)
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
