"""The seeded input generators: determinism, shape, canonical order."""
import numpy as np
import pytest
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


@pytest.mark.gpu
@pytest.mark.parametrize("name,scale", [("er_tiny", 1.0), ("rmat_dense_wide", 0.01), ("rmat_sparse_stack", 0.004),
                                        ("rmat_weighted_narrow", 0.02), ("rmat_capacity", 0.0002)])
def test_generators_give_the_same_graph_on_cpu_and_gpu(name, scale):
    """Every random bit comes from integer counters, so the device must not matter: the oracle side
    (CPU tensors) and the HIP side (GPU tensors) of a parity test see the same edges."""
    a = synth.make_graph(name, scale=scale)
    b = synth.make_graph(name, scale=scale, device=torch.device("cuda:0"))
    assert (a.n, a.e) == (b.n, b.e)
    assert torch.equal(a.src, b.src.cpu()) and torch.equal(a.dst, b.dst.cpu())
    # Features pass through log / cos, whose last bit may differ between the two math libraries:
    # the parity tests therefore generate a matrix once and hand the same bits to both sides.
    x = synth.make_features(name, 257, 33, 9)
    y = synth.make_features(name, 257, 33, 9, device=torch.device("cuda:0"))
    assert torch.allclose(x.float(), y.cpu().float(), rtol=1e-2 if x.dtype == torch.bfloat16 else 1e-5, atol=1e-6)
    if synth.WORKLOADS[name].get("weighted"):
        wa = synth.gcn_sym_edge_weights(a.dst, a.src, a.n)
        wb = synth.gcn_sym_edge_weights(b.dst, b.src, b.n)
        assert torch.equal(wa, wb.cpu())


@pytest.mark.parametrize("kind", ["degree", "rmat_prefix", "random"])
def test_relabel_keeps_the_graph(kind):
    """A vertex reordering renames vertices and nothing else: same edge count, same degree
    multiset, canonical order, still symmetric; the degree order really is by descending degree."""
    el = synth.make_graph("rmat_sparse_stack", scale=0.002)
    r = synth.relabel(el, kind, seed=3)
    assert (r.n, r.e) == (el.n, el.e) and _canonical(r)
    d0 = torch.bincount(el.dst.long(), minlength=el.n)
    d1 = torch.bincount(r.dst.long(), minlength=el.n)
    assert torch.equal(torch.sort(d0).values, torch.sort(d1).values)
    assert torch.equal(d1, torch.bincount(r.src.long(), minlength=el.n))  # symmetric graph stays symmetric
    if kind == "degree":
        assert bool((d1[1:] <= d1[:-1]).all())
    from synth.graphs import _scramble, _unscramble
    x = torch.arange(1 << 13, dtype=torch.int64)
    assert torch.equal(_unscramble(_scramble(x, 13, 7), 13, 7), x)
