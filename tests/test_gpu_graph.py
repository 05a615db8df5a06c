"""The entry points allocate nothing and only enqueue kernels on the caller's stream, so a
training-style sequence (sampling forward, zero-fill of the gradient table, backward) can be
captured into a HIP graph and replayed.  Each replay, with new seeds copied into the captured
input buffer and eager work in between, must reproduce the eager result: IDs and forward
outputs bit for bit, the gradient table to the backward's tolerance."""
import numpy as np
import pytest
import torch

from test_gpu_parity import ragged_graph

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("fan", [[15], [15, 10]])
def test_forward_backward_under_graph_capture(fan):
    from paper_2511_13645_amd import binding as fsa
    n, D, B = 5000, 128, 1024
    indptr, indices = ragged_graph(n, seed=21)
    d_indptr, d_indices = torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV)
    rng = np.random.default_rng(1)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(DEV)
    g = torch.from_numpy(rng.standard_normal((B, D)).astype(np.float32)).to(DEV)
    two = len(fan) == 2
    k1, k2 = fan[0], (fan[1] if two else 0)

    # static buffers of the captured graph
    seeds = torch.zeros(B, dtype=torch.int32, device=DEV)
    out = torch.empty((B, D), device=DEV)
    h1 = torch.empty((B, k1, D), device=DEV) if two else None
    ids1 = torch.empty((B, k1), dtype=torch.int32, device=DEV)
    ids2 = torch.empty((B, k1, k2), dtype=torch.int32, device=DEV) if two else None
    gx = torch.empty((n, D), device=DEV)

    def step():
        fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, fan, 5, out=out, out_h1=h1, out_ids1=ids1, out_ids2=ids2)
        gx.zero_()                                     # a fill kernel, not a memset node
        fsa.fsa_mean_bwd(g, ids1, ids2, grad_x=gx)

    batches = [torch.from_numpy(rng.integers(0, n, B).astype(np.int32)).to(DEV) for _ in range(4)]
    seeds.copy_(batches[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside capture, as torch asks
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i, batch in enumerate(batches):
        seeds.copy_(batch)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (out, ids1, gx)] + ([h1.clone(), ids2.clone()] if two else [])
        # eager reference with fresh buffers, and unrelated eager work between replays
        e_out, e_h1, e_ids1, e_ids2 = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, batch, fan, 5)
        e_gx = fsa.fsa_mean_bwd(g, e_ids1, e_ids2, grad_x=torch.zeros((n, D), device=DEV))
        torch.cuda.synchronize()
        assert torch.equal(got[0], e_out) and torch.equal(got[1], e_ids1), "replay %d" % i
        if two:
            assert torch.equal(got[3], e_h1) and torch.equal(got[4], e_ids2), "replay %d" % i
        assert torch.allclose(got[2], e_gx, rtol=1e-5, atol=1e-6), "replay %d" % i
        assert (got[2] != 0).any()
