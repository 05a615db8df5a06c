"""1-hop calls of 32768 seeds and more take several seeds per wave (the 2-hop kernel with the
seeds as its slots).  Same comparisons as the small-batch parity tests --
IDs bit-exact, means and gradients within tolerance of the oracle, emission-off and replay
bitwise equal -- at batch sizes on both sides of the switch and not a multiple of the seeds
per wave, so the last wave has missing seeds."""
import numpy as np
import pytest
import torch

from parity_util import TOL, assert_close, assert_ids_equal, forward_scales, host_x, to_f64
from test_gpu_parity import ragged_graph, run_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("k", [1, 2, 7, 10, 15, 16, 21, 32])
def test_large_batch_one_hop_fp32(fsa, orc, k):
    n, D = 3000, 24
    indptr, indices = ragged_graph(n, seed=k, max_deg=40)
    x = torch.from_numpy(np.random.default_rng(k).standard_normal((n, D)).astype(np.float32))
    rng = np.random.default_rng(7)
    B = (32768 if k % 2 else 70000) + 1 + int(rng.integers(0, 3000))    # ragged: not a multiple of the seeds per wave
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, [k], 40 + k, what="large-batch 1-hop k=%d B=%d" % (k, B))


@pytest.mark.parametrize("D,dtype", [(1, torch.float32), (100, torch.float32), (128, torch.bfloat16), (130, torch.bfloat16),
                                     (257, torch.float32), (602, torch.float32), (1000, torch.float32)])
def test_large_batch_one_hop_row_shapes(fsa, orc, D, dtype):
    """Every row geometry (chunk widths 16/8/4/2, one tile, several tiles) and int64 indptr."""
    n, k = 1500, 15
    indptr, indices = ragged_graph(n, seed=D, max_deg=30, wide=True)
    x = torch.from_numpy(np.random.default_rng(D).standard_normal((n, D)).astype(np.float32)).to(dtype)
    rng = np.random.default_rng(D)
    B = 32771 if D > 300 else 40001
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    run_case(fsa, orc, indptr, indices, x, seeds, [k], 5, check_bwd=(dtype == torch.float32 and D <= 257),
             what="large-batch 1-hop D=%d %s" % (D, dtype))


def test_same_ids_and_means_on_both_sides_of_the_switch(fsa):
    """A seed's IDs and mean do not depend on the batch it is in: the first seeds of a large batch
    (several seeds per wave) equal the same seeds run as a small batch (a wave per seed)."""
    n, D, k = 4000, 64, 15
    indptr, indices = ragged_graph(n, seed=3, max_deg=60)
    dev = "cuda:0"
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    x = torch.randn((n, D), generator=torch.Generator().manual_seed(1)).to(dev)
    seeds = torch.from_numpy(np.random.default_rng(0).integers(0, n, 50000).astype(np.int32)).to(dev)
    big = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, [k], 11)
    small = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds[:3000].contiguous(), [k], 11)
    torch.cuda.synchronize()
    assert torch.equal(big[2][:3000], small[2])
    assert torch.allclose(big[0][:3000], small[0], rtol=2e-6, atol=1e-6)


def test_large_batch_weighted_one_hop(fsa, orc):
    n, D, k = 2500, 40, 10
    rng = np.random.default_rng(5)
    indptr, indices = ragged_graph(n, seed=9, max_deg=35)
    ew = rng.random(indices.size).astype(np.float32)
    ew[rng.random(indices.size) < 0.1] = 0.0
    ew[indptr[20]:indptr[21]] = 0.0                                # a row whose weights are all zero
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    B = 34567
    seeds = np.concatenate([np.arange(24), rng.integers(0, n, B - 24)]).astype(np.int32)
    dev = "cuda:0"
    r_out, _, r_ids1, _, r_w1, _ = orc.sample_wmean_fwd(indptr, indices, ew, x.numpy(), seeds, [k], 3)
    d_x = x.to(dev)
    out, _, ids1, _, w1, _ = fsa.fsa_sample_wmean_fwd(torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev),
                                                      torch.from_numpy(ew).to(dev), d_x, torch.from_numpy(seeds).to(dev), [k], 3)
    torch.cuda.synchronize()
    assert_ids_equal(ids1, r_ids1, "ids1")
    assert np.array_equal(w1.cpu().numpy(), r_w1)
    m = (ids1 >= 0).float() * w1
    a = ((d_x.abs()[ids1.clamp(min=0).long()] * m[..., None]).sum(1) / m.sum(1).clamp(min=1e-30)[:, None]).double().cpu().numpy()
    assert_close(to_f64(out), r_out, a, 1e-5, "weighted out")
    rp, _ = fsa.fsa_wmean_replay_fwd(d_x, ids1, w1)
    torch.cuda.synchronize()
    assert torch.equal(rp, out)


def test_large_batch_with_negative_seeds_and_saved_ids_with_holes(fsa, orc):
    """Replay of a large 1-hop batch whose saved IDs have holes anywhere, including whole empty rows."""
    n, D, k = 2000, 32, 12
    rng = np.random.default_rng(2)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    B = 45678
    ids1 = rng.integers(0, n, (B, k)).astype(np.int32)
    ids1[rng.random((B, k)) < 0.3] = -1
    ids1[::17] = -1
    ref, _ = orc.mean_replay_fwd(x.numpy(), ids1)
    dev = "cuda:0"
    d_ids = torch.from_numpy(ids1).to(dev)
    out, _ = fsa.fsa_mean_replay_fwd(x.to(dev), d_ids)
    torch.cuda.synchronize()
    a, _ = forward_scales(x.to(dev), d_ids, None)
    assert_close(to_f64(out), ref, a, 1e-5, "replay with holes")
    assert float(out[::17].abs().sum()) == 0.0


@pytest.mark.parametrize("B", [32769, 40003, 65537])
def test_last_wave_writes_nothing_beyond_the_batch(fsa, B):
    """Outputs carved out of larger buffers with sentinel words on both sides: the last wave's
    missing seeds (B is not a multiple of the seeds per wave) leave the sentinels alone, and the
    carved outputs equal those of an ordinary call."""
    n, D, k, G = 3000, 32, 15, 4096
    indptr, indices = ragged_graph(n, seed=B % 97, max_deg=40)
    dev = "cuda:0"
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    x = torch.randn((n, D), generator=torch.Generator().manual_seed(2)).to(dev)
    seeds = torch.from_numpy(np.random.default_rng(B).integers(0, n, B).astype(np.int32)).to(dev)
    want = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, [k], 19)
    buf_out = torch.full((G + B * D + G,), -7.5, dtype=torch.float32, device=dev)
    buf_ids = torch.full((G + B * k + G,), -12345, dtype=torch.int32, device=dev)
    out = buf_out[G:G + B * D].view(B, D)
    ids = buf_ids[G:G + B * k].view(B, k)
    fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, [k], 19, out=out, out_ids1=ids)
    torch.cuda.synchronize()
    assert torch.equal(out, want[0]) and torch.equal(ids, want[2])
    for buf, fill in ((buf_out, -7.5), (buf_ids, -12345)):
        assert bool((buf[:G] == fill).all()) and bool((buf[-G:] == fill).all())
    # replay from the carved IDs, outputs carved again
    buf_out.fill_(-7.5)
    fsa.fsa_mean_replay_fwd(x, ids, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out, want[0])
    assert bool((buf_out[:G] == -7.5).all()) and bool((buf_out[-G:] == -7.5).all())
