"""The seeded input generators: determinism, shape, canonical order."""
import numpy as np
import torch

import synth


def _canonical(el):
    key = el.dst.long() * el.n + el.src.long()
    return bool((key[1:] > key[:-1]).all())


def test_er_tiny_shape_and_determinism():
    a = synth.make_graph("er_tiny")
    b = synth.make_graph("er_tiny")
    assert (a.n, a.e) == (4096, 65536)
    assert torch.equal(a.src, b.src) and torch.equal(a.dst, b.dst)
    assert _canonical(a) and bool((a.src != a.dst).all())
    c = synth.make_graph("er_tiny", seed=1)
    assert not torch.equal(a.src, c.src)


def test_rmat_symmetric_is_symmetric_and_skewed():
    el = synth.make_graph("rmat_sparse_stack", scale=0.004)
    assert _canonical(el) and el.e % 2 == 0 and bool((el.src != el.dst).all())
    fwd = set(zip(el.src.tolist(), el.dst.tolist()))
    assert all((d, s) in fwd for s, d in list(fwd)[:5000])
    deg = torch.bincount(el.dst.long(), minlength=el.n)
    assert abs(deg.float().mean().item() - 123718280 / 2449029) < 0.1
    assert deg.max().item() > 20 * deg.float().mean().item()      # power-law tail
    assert int(deg.min()) == 0                                    # and isolated vertices


def test_rmat_directed_exact_edge_count():
    el = synth.make_graph("rmat_capacity", scale=0.0002)
    assert el.e == round(1615685872 * 0.0002) and _canonical(el)
    rev = set(zip(el.dst.tolist(), el.src.tolist()))
    fwd = set(zip(el.src.tolist(), el.dst.tolist()))
    assert len(fwd & rev) < 0.5 * len(fwd)                        # genuinely directed


def test_features_are_seeded_and_distributed():
    x = synth.normal_features(4000, 50, 3)
    assert torch.equal(x, synth.normal_features(4000, 50, 3, chunk_rows=777))
    assert abs(x.mean().item()) < 0.01 and abs(x.std().item() - 1.0) < 0.01
    u = synth.uniform_features(4000, 50, 3)
    assert u.min().item() >= -1.0 and u.max().item() < 1.0 and abs(u.mean().item()) < 0.01
    b = synth.normal_features(100, 8, 3, dtype=torch.bfloat16)
    assert b.dtype == torch.bfloat16


def test_gcn_edge_weights():
    el = synth.make_graph("rmat_weighted_narrow", scale=0.02)
    w = synth.gcn_sym_edge_weights(el.dst, el.src, el.n)
    deg = np.bincount(el.dst.numpy(), minlength=el.n).astype(np.float64)
    ref = 1.0 / np.sqrt(deg[el.src.numpy()] * deg[el.dst.numpy()])
    assert np.allclose(w.numpy(), ref.astype(np.float32))
