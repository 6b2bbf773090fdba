"""Pins of the layer oracle (oracle/layer_oracle.c): dense product, one GraphSAGE layer and
its gradients, against things other than itself; planted mistakes must trip a pin."""
from __future__ import annotations

import os
import tempfile

import numpy as np
import pytest

import oracle
import synth


def small_graph(n, e, seed):
    el = synth.small_random_multigraph(n, e, seed)
    dst, src = synth.to_csr_numpy(el)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(indptr, dst.astype(np.int64) + 1, 1)
    return np.cumsum(indptr), src.astype(np.int32), dst.astype(np.int64)


def dense_operator(indptr, src, dst, n):
    """(A + I) / (din + 1) as a dense matrix."""
    A = np.zeros((n, n))
    np.add.at(A, (dst, src.astype(np.int64)), 1.0)
    A += np.eye(n)
    return A / (np.diff(indptr)[:, None] + 1.0)


def pin_matmul_is_numpy_matmul():
    rng = np.random.default_rng(1)
    for (m, n, k) in ((1, 1, 1), (5, 3, 7), (17, 33, 9), (8, 8, 0), (40, 2, 64)):
        for ta in (False, True):
            for tb in (False, True):
                A = rng.normal(size=(k, m) if ta else (m, k)).astype(np.float32)
                B = rng.normal(size=(n, k) if tb else (k, n)).astype(np.float32)
                bias = rng.normal(size=n).astype(np.float32)
                a64 = (A.T if ta else A).astype(np.float64)
                b64 = (B.T if tb else B).astype(np.float64)
                for use_bias in (False, True):
                    for relu in (False, True):
                        C, S = oracle.matmul(A, B, ta, tb, bias if use_bias else None, relu)
                        ref = a64 @ b64 + (bias.astype(np.float64) if use_bias else 0.0)
                        mag = np.abs(a64) @ np.abs(b64) + (np.abs(bias.astype(np.float64)) if use_bias else 0.0)
                        if relu:
                            ref = np.maximum(ref, 0.0)
                        assert np.allclose(C, ref, rtol=1e-13, atol=1e-13), (m, n, k, ta, tb, use_bias, relu)
                        assert np.allclose(S, mag, rtol=1e-13, atol=1e-13)
    # not symmetric in its operands, and a transpose flag is not a no-op
    A = np.arange(6, dtype=np.float32).reshape(2, 3)
    B = np.arange(6, dtype=np.float32).reshape(3, 2) + 1
    C, _ = oracle.matmul(A, B)
    assert C.tolist() == [[13.0, 16.0], [40.0, 52.0]]
    C, _ = oracle.matmul(B, A, trans_a=True, trans_b=True)
    assert C.tolist() == (B.T.astype(np.float64) @ A.T.astype(np.float64)).tolist()


def pin_layer_forward_is_dense_algebra():
    rng = np.random.default_rng(2)
    for case, (n, e, fi, fo) in enumerate(((1, 1, 3, 2), (9, 30, 4, 6), (30, 200, 7, 3), (12, 5, 2, 2))):
        indptr, src, dst = small_graph(n, e, 40 + case)
        X = rng.normal(size=(n, fi)).astype(np.float32)
        W = rng.normal(size=(fi, fo)).astype(np.float32)
        b = rng.normal(size=fo).astype(np.float32)
        Ahat = dense_operator(indptr, src, dst, n)
        for bias in (None, b):
            for relu in (False, True):
                Z, H, SH = oracle.sage_layer_fwd(indptr, src, X, W, bias, relu)
                zref = Ahat @ X.astype(np.float64)
                href = zref @ W.astype(np.float64) + (0.0 if bias is None else bias.astype(np.float64))
                if relu:
                    href = np.maximum(href, 0.0)
                assert np.allclose(Z, zref, rtol=1e-12, atol=1e-12)
                assert np.allclose(H, href, rtol=1e-12, atol=1e-12), (case, bias is None, relu)
                sref = (Ahat @ np.abs(X.astype(np.float64))) @ np.abs(W.astype(np.float64)) + \
                    (0.0 if bias is None else np.abs(bias.astype(np.float64)))
                assert np.allclose(SH, sref, rtol=1e-12, atol=1e-12)
                # the aggregation step is the aggregation oracle's SAGE_GCN
                assert np.allclose(Z, oracle.aggregate_fwd(indptr, src, X, op=oracle.OP_SAGE_GCN), rtol=1e-12, atol=1e-12)
                # the order of the two linear steps does not matter
                if not relu and bias is None:
                    P, _ = oracle.matmul(X, W)
                    assert np.allclose(H, Ahat @ P, rtol=1e-11, atol=1e-11)


def pin_layer_closed_forms():
    # no edges: every vertex aggregates only itself -> a plain dense layer
    n, fi, fo = 5, 3, 4
    rng = np.random.default_rng(3)
    X = rng.normal(size=(n, fi)).astype(np.float32)
    W = rng.normal(size=(fi, fo)).astype(np.float32)
    indptr = np.zeros(n + 1, dtype=np.int64)
    src = np.zeros(0, dtype=np.int32)
    _, H, _ = oracle.sage_layer_fwd(indptr, src, X, W, None, False)
    assert np.allclose(H, X.astype(np.float64) @ W.astype(np.float64), rtol=1e-13, atol=1e-13)
    # identity weights, all-ones features on any graph: (din + 1) / (din + 1) = 1
    indptr, src, dst = small_graph(20, 90, 4)
    _, H, _ = oracle.sage_layer_fwd(indptr, src, np.ones((20, 3), np.float32), np.eye(3, dtype=np.float32), None, True)
    assert np.allclose(H, 1.0, rtol=1e-13, atol=1e-13)
    # the rectifier clamps, the bias shifts
    _, H, _ = oracle.sage_layer_fwd(indptr, src, np.ones((20, 3), np.float32), -np.eye(3, dtype=np.float32),
                                    np.array([0.5, 1.0, 2.0], np.float32), True)
    assert np.allclose(H, np.array([0.0, 0.0, 1.0]), rtol=1e-13, atol=1e-13)


def pin_layer_gradients_by_finite_differences():
    rng = np.random.default_rng(5)
    n, fi, fo = 7, 3, 4
    indptr, src, dst = small_graph(n, 18, 6)
    Ahat = dense_operator(indptr, src, dst, n)
    X = rng.normal(size=(n, fi)).astype(np.float32)
    W = rng.normal(size=(fi, fo)).astype(np.float32)
    b = rng.normal(size=fo).astype(np.float32)
    dH = rng.normal(size=(n, fo)).astype(np.float32)
    h = 1e-6
    for relu in (False, True):
        _, H, _ = oracle.sage_layer_fwd(indptr, src, X, W, b, relu)
        Hs = H.astype(np.float32)
        assert not relu or np.abs(Ahat @ X.astype(np.float64) @ W.astype(np.float64) + b).min() > 1e-3  # no kink nearby

        def loss(x64, w64, b64):
            out = Ahat @ x64 @ w64 + b64
            if relu:
                out = np.maximum(out, 0.0)
            return float((out * dH.astype(np.float64)).sum())
        g = oracle.sage_layer_bwd(indptr, src, X, W, Hs, dH, relu)
        base = [X.astype(np.float64), W.astype(np.float64), b.astype(np.float64)]
        for which, key in ((0, "dX"), (1, "dW"), (2, "db")):
            num = np.zeros_like(base[which])
            for idx in np.ndindex(*base[which].shape):
                p = [a.copy() for a in base]
                m = [a.copy() for a in base]
                p[which][idx] += h
                m[which][idx] -= h
                num[idx] = (loss(*p) - loss(*m)) / (2 * h)
            val, mag = g[key]
            assert np.allclose(val, num, rtol=1e-5, atol=1e-7), (relu, key)
            assert (mag >= np.abs(val) - 1e-12).all()


def pin_layer_gradients_are_dense_algebra():
    rng = np.random.default_rng(7)
    n, fi, fo = 25, 5, 6
    indptr, src, dst = small_graph(n, 140, 8)
    Ahat = dense_operator(indptr, src, dst, n)
    X = rng.normal(size=(n, fi)).astype(np.float32)
    W = rng.normal(size=(fi, fo)).astype(np.float32)
    dH = rng.normal(size=(n, fo)).astype(np.float32)
    Hs = rng.normal(size=(n, fo)).astype(np.float32)  # any stored output: only its sign matters
    g = oracle.sage_layer_bwd(indptr, src, X, W, Hs, dH, True)
    G = np.where(Hs > 0, dH, 0).astype(np.float64)
    Z = Ahat @ X.astype(np.float64)
    assert np.allclose(g["db"][0], G.sum(0), rtol=1e-12, atol=1e-12)
    assert np.allclose(g["dW"][0], Z.T @ G, rtol=1e-12, atol=1e-12)
    assert np.allclose(g["dX"][0], Ahat.T @ (G @ W.astype(np.float64).T), rtol=1e-12, atol=1e-12)
    assert np.allclose(g["db"][1], np.abs(G).sum(0), rtol=1e-12, atol=1e-12)
    assert np.allclose(g["dW"][1], (Ahat @ np.abs(X.astype(np.float64))).T @ np.abs(G), rtol=1e-12, atol=1e-12)
    assert np.allclose(g["dX"][1], Ahat.T @ (np.abs(G) @ np.abs(W.astype(np.float64)).T), rtol=1e-12, atol=1e-12)


PINS = [pin_matmul_is_numpy_matmul, pin_layer_forward_is_dense_algebra, pin_layer_closed_forms,
        pin_layer_gradients_by_finite_differences, pin_layer_gradients_are_dense_algebra]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin()


MUTATIONS = [
    ("matmul_transpose_a_ignored", "double a = trans_a ? (double)A[k * lda + m] : (double)A[m * lda + k];", "double a = (double)A[m * lda + k];"),
    ("matmul_transpose_b_swapped", "double b = trans_b ? (double)B[n * ldb + k] : (double)B[k * ldb + n];", "double b = trans_b ? (double)B[k * ldb + n] : (double)B[n * ldb + k];"),
    ("matmul_bias_by_row", "acc += (double)bias[n];\n                mag += fabs((double)bias[n]);", "acc += (double)bias[m % N];\n                mag += fabs((double)bias[n]);"),
    ("matmul_relu_missing", "if (relu && acc < 0.0) acc = 0.0;\n            C[m * N + n] = acc;", "C[m * N + n] = acc;"),
    ("layer_self_term_dropped", "double x = (double)X[v * Fi + k];\n            z[k] = x;", "double x = (double)X[v * Fi + k];\n            z[k] = 0.0;"),
    ("layer_divides_by_din", "z[k] /= din + 1.0;\n            sz[k] /= din + 1.0;", "z[k] /= (din > 0 ? din : 1.0);\n            sz[k] /= din + 1.0;"),
    ("layer_weight_transposed", "acc += z[k] * (double)W[k * Fo + j];", "acc += z[k] * (double)W[j * Fi + k];"),
    ("layer_relu_before_bias", "if (bias) {\n                acc += (double)bias[j];\n                mag += fabs((double)bias[j]);\n            }\n            if (relu && acc < 0.0) acc = 0.0;\n            H[v * Fo + j] = acc;",
     "if (relu && acc < 0.0) acc = 0.0;\n            if (bias) {\n                acc += (double)bias[j];\n                mag += fabs((double)bias[j]);\n            }\n            H[v * Fo + j] = acc;"),
    ("bwd_mask_ignored", "double pass = (!relu || Hs[v * Fo + j] > 0.0f) ? 1.0 : 0.0;", "double pass = 1.0;"),
    ("bwd_mask_from_gradient", "double pass = (!relu || Hs[v * Fo + j] > 0.0f) ? 1.0 : 0.0;", "double pass = (!relu || dH[v * Fo + j] > 0.0f) ? 1.0 : 0.0;"),
    ("bwd_dw_uses_raw_input", "dW[k * Fo + j] += z[k] * g[j];", "dW[k * Fo + j] += (double)X[v * Fi + k] * g[j];"),
    ("bwd_dz_unscaled", "dz[k] = acc * scale;", "dz[k] = acc;"),
    ("bwd_self_gradient_dropped", "dX[v * Fi + k] += dz[k];", "dX[v * Fi + k] += 0.0;"),
    ("bwd_scatter_to_destination", "int64_t u = indices[e];\n            for (int64_t k = 0; k < Fi; ++k) {\n                dX[u * Fi + k] += dz[k];", "int64_t u = v;\n            for (int64_t k = 0; k < Fi; ++k) {\n                dX[u * Fi + k] += dz[k];"),
    ("bwd_dz_weight_index", "acc += g[j] * (double)W[k * Fo + j];\n                mag", "acc += g[j] * (double)W[(k * Fo + j + 1) % (Fi * Fo)];\n                mag"),
]


@pytest.mark.parametrize("mutation", MUTATIONS, ids=lambda m: m[0])
def test_pins_catch_planted_mistakes(mutation):
    name, old, new = mutation
    src_dir = os.path.dirname(oracle.__file__)
    text = open(os.path.join(src_dir, "layer_oracle.c")).read()
    assert text.count(old) == 1, f"mutation {name}: anchor text must occur exactly once"
    with tempfile.TemporaryDirectory() as tmp:
        c_path = os.path.join(tmp, "mutant_layer.c")
        so_path = os.path.join(tmp, f"mutant_{name}.so")
        with open(c_path, "w") as fh:
            fh.write(text.replace(old, new))
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
