"""The synthetic-input recipes: determinism, CSR validity and the advertised shapes (no GPU)."""
import numpy as np
import torch

from paper_2511_13645_amd import synth


def _check_csr(g):
    ip = g.indptr.to(torch.int64)
    assert ip[0] == 0 and ip[-1] == g.num_edges and (ip[1:] >= ip[:-1]).all()
    assert g.indices.dtype == torch.int32
    if g.num_edges:
        assert g.indices.min() >= 0 and g.indices.max() < g.num_nodes


def test_tiny_graph_has_every_degree_regime():
    g = synth.tiny_graph()
    _check_csr(g)
    d = g.degrees()
    assert g.num_nodes == 10_000 and d.max() == 200
    for want in (0, 1, 9, 10, 11):
        assert (d == want).any()
    src = torch.repeat_interleave(torch.arange(g.num_nodes), d)
    assert (src != g.indices).all()                      # no self-loops
    g2 = synth.tiny_graph()
    assert torch.equal(g.indices, g2.indices) and torch.equal(g.indptr, g2.indptr)


def test_chung_lu_shape_and_determinism():
    g = synth.chung_lu_graph(50_000, 40.0, 3000.0, seed=0)
    _check_csr(g)
    d = g.degrees().double()
    assert abs(d.mean().item() - 40.0) < 2.0
    assert 2500 <= d.max().item() <= 3001
    assert 0.005 < (d == 0).double().mean().item() < 0.02
    # heavy tail: the top 1% of rows own far more than 1% of the edges
    top = torch.sort(d, descending=True).values[:500].sum() / d.sum()
    assert top > 0.08
    # popular targets: in-degree is heavy-tailed too and correlates with out-degree
    indeg = torch.bincount(g.indices.long(), minlength=g.num_nodes).double()
    assert np.corrcoef(indeg.numpy(), d.numpy())[0, 1] > 0.5
    src = torch.repeat_interleave(torch.arange(g.num_nodes), g.degrees())
    assert (src != g.indices).all()
    h = synth.chung_lu_graph(50_000, 40.0, 3000.0, seed=0, edge_chunk=100_000)
    assert torch.equal(g.indices, h.indices) and torch.equal(g.indptr, h.indptr)   # chunking is invisible
    k = synth.chung_lu_graph(50_000, 40.0, 3000.0, seed=1)
    assert not torch.equal(g.indptr, k.indptr)
    w = synth.chung_lu_graph(5_000, 10.0, 300.0, seed=0, wide_indptr=True)
    assert w.indptr.dtype == torch.int64


def test_kg_graph_is_symmetric_with_a_hub():
    g = synth.kg_graph(20_000, 130_000, seed=0)
    _check_csr(g)
    assert g.num_edges == 260_000
    d = g.degrees()
    assert d.max().item() > 0.05 * g.num_edges            # Zipf(1.1) head entity
    src = torch.repeat_interleave(torch.arange(g.num_nodes), d)
    fwd = torch.sort(src * g.num_nodes + g.indices.long()).values
    bwd = torch.sort(g.indices.long() * g.num_nodes + src).values
    assert torch.equal(fwd, bwd)                          # both directions stored


def test_features_and_batches():
    x = synth.features(4000, 16, seed=1)
    assert abs(x.mean().item()) < 0.02 and abs(x.std().item() - 1.0) < 0.02
    assert torch.equal(x, synth.features(4000, 16, seed=1, chunk_rows=77))
    u = synth.features(4000, 8, dist="uniform", scale=0.1, seed=1)
    assert u.min() >= -0.1 and u.max() <= 0.1 and abs(u.mean().item()) < 0.01
    b = synth.features(100, 8, dtype=torch.bfloat16)
    assert b.dtype == torch.bfloat16
    s = synth.seed_batches(1000, 64, 3)
    assert s.shape == (3, 64) and s.dtype == torch.int32
    for row in s:
        assert len(set(row.tolist())) == 64
    assert synth.upstream_grad((5, 7)).shape == (5, 7)


def test_scaled_workloads_build():
    for name in ("products", "social", "kg", "citation"):
        w = synth.make_workload(name, scale=0.002 if name != "social" else 0.02)
        _check_csr(w.graph)
        assert w.x.shape[0] == w.graph.num_nodes
    w = synth.make_workload("citation", scale=0.0005)
    assert w.graph.indptr.dtype == torch.int64 and w.x.dtype == torch.bfloat16
