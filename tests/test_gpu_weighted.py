"""GPU parity of the weighted-mean entry points against the oracle's weighted functions."""
import numpy as np
import pytest
import torch

from parity_util import TOL, assert_close, assert_ids_equal, host_x, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    return binding


def _graph(n, seed, max_deg=90, wide=False):
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, max_deg + 1, size=n)
    deg[rng.random(n) < 0.15] = 0
    deg[:8] = [0, 1, 9, 10, 11, 64, 65, 3000]
    indptr = np.concatenate([[0], np.cumsum(deg)])
    indices = rng.integers(0, n, size=int(indptr[-1])).astype(np.int32)
    ew = rng.random(indices.size).astype(np.float32)
    ew[rng.random(indices.size) < 0.1] = 0.0                        # some zero weights
    ew[indptr[20]:indptr[21]] = 0.0                                 # a row whose weights are all zero
    return indptr.astype(np.int64 if wide else np.int32), indices, ew


def _scales(x, ids1, ids2, w1, w2):
    """A for the weighted means: weighted mean of |x| over the same rows (on the device)."""
    xa = x.float().abs()
    if ids2 is None:
        m = (ids1 >= 0).float() * w1
        num = (xa[ids1.clamp(min=0).long()] * m[..., None]).sum(1)
        return (num / m.sum(1).clamp(min=1e-30)[:, None]).double().cpu().numpy(), None
    m2 = (ids2 >= 0).float() * w2
    num = (xa[ids2.clamp(min=0).long()] * m2[..., None]).sum(2)
    a_h1 = num / m2.sum(2).clamp(min=1e-30)[..., None]
    part = ((m2.sum(2) > 0) & (ids1 >= 0)).float() * w1
    a_out = (a_h1 * part[..., None]).sum(1) / part.sum(1).clamp(min=1e-30)[:, None]
    return a_out.double().cpu().numpy(), a_h1.double().cpu().numpy()


def _run(fsa, orc, indptr, indices, ew, x, seeds, fan, seed, what, check_bwd=True):
    dev = "cuda:0"
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    d_ew, d_x, d_seeds = torch.from_numpy(ew).to(dev), x.to(dev), torch.from_numpy(seeds).to(dev)
    tol = 1e-3 if x.dtype == torch.float16 else TOL[x.dtype]     # fp16: one rounding, half an ulp = 2^-11
    hx, is_bf16 = (x.to(torch.float64).numpy(), False) if x.dtype == torch.float16 else host_x(x)
    r_out, r_h1, r_ids1, r_ids2, r_w1, r_w2 = orc.sample_wmean_fwd(indptr, indices, ew, hx, seeds, fan, seed, bf16=is_bf16)
    out, h1, ids1, ids2, w1, w2 = fsa.fsa_sample_wmean_fwd(d_indptr, d_indices, d_ew, d_x, d_seeds, fan, seed)
    torch.cuda.synchronize()
    assert_ids_equal(ids1, r_ids1, what + " ids1")
    assert np.array_equal(w1.cpu().numpy(), r_w1), what + " w1"
    if len(fan) == 2:
        assert_ids_equal(ids2, r_ids2, what + " ids2")
        assert np.array_equal(w2.cpu().numpy(), r_w2), what + " w2"
    # the sampler is the unweighted one: same IDs for the same seed
    u = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, d_x, d_seeds, fan, seed, emit_h1=False)
    assert torch.equal(u[2], ids1) and (len(fan) == 1 or torch.equal(u[3], ids2))
    a_out, a_h1 = _scales(d_x, ids1, ids2, w1, w2)
    assert_close(to_f64(out), r_out, a_out, tol, what + " out")
    if len(fan) == 2:
        assert_close(to_f64(h1), r_h1, a_h1, tol, what + " out_h1")
    rp_out, rp_h1 = fsa.fsa_wmean_replay_fwd(d_x, ids1, w1, ids2, w2)
    torch.cuda.synchronize()
    assert torch.equal(rp_out.view(torch.uint8), out.view(torch.uint8)), what + " replay out differs"
    if len(fan) == 2:
        assert torch.equal(rp_h1.view(torch.uint8), h1.view(torch.uint8)), what + " replay h1 differs"
    if check_bwd:
        B, D, N = seeds.shape[0], x.shape[1], x.shape[0]
        rng = np.random.default_rng(3)
        g = torch.from_numpy(rng.standard_normal((B, D)).astype(np.float32)).to(dev)
        gh = torch.from_numpy(rng.standard_normal((B, fan[0], D)).astype(np.float32)).to(dev) if len(fan) == 2 else None
        gx = torch.zeros((N, D), dtype=torch.float32, device=dev)
        fsa.fsa_wmean_bwd(g, ids1, w1, ids2, w2, gh, grad_x=gx)
        torch.cuda.synchronize()
        ghn = None if gh is None else to_f64(gh)
        r_gx = orc.wmean_bwd(to_f64(g), r_ids1, r_w1, r_ids2, r_w2, ghn, num_nodes=N)
        scale = orc.wmean_bwd(np.abs(to_f64(g)), r_ids1, r_w1, r_ids2, r_w2, None if ghn is None else np.abs(ghn), num_nodes=N)
        assert_close(to_f64(gx), r_gx, scale, 1e-5, what + " grad_x")


@pytest.mark.parametrize("D", [1, 6, 64, 100, 128, 257, 260, 602, 1000, 2052])
@pytest.mark.parametrize("fan", [[10], [15, 10]])
def test_weighted_fp32(fsa, orc, D, fan):
    n = 2500
    indptr, indices, ew = _graph(n, seed=D)
    x = torch.from_numpy(np.random.default_rng(D).standard_normal((n, D)).astype(np.float32))
    seeds = np.concatenate([np.arange(24), np.random.default_rng(1).integers(0, n, 233)]).astype(np.int32)
    _run(fsa, orc, indptr, indices, ew, x, seeds, fan, 77 + D, "weighted fp32 D=%d fan=%s" % (D, fan))


@pytest.mark.parametrize("D", [3, 128, 200, 520, 2056])
@pytest.mark.parametrize("fan", [[15], [25, 10], [3, 33]])
def test_weighted_bf16_wide_indptr(fsa, orc, D, fan):
    n = 2000
    indptr, indices, ew = _graph(n, seed=50 + D, wide=True)
    x = torch.from_numpy(np.random.default_rng(D).standard_normal((n, D)).astype(np.float32)).to(torch.bfloat16)
    seeds = np.concatenate([np.arange(24), np.random.default_rng(2).integers(0, n, 150)]).astype(np.int32)
    _run(fsa, orc, indptr, indices, ew, x, seeds, fan, 5, "weighted bf16 D=%d fan=%s" % (D, fan), check_bwd=False)


@pytest.mark.parametrize("D", [2, 128, 330])
@pytest.mark.parametrize("fan", [[15], [15, 10]])
def test_weighted_fp16(fsa, orc, D, fan):
    n = 2000
    indptr, indices, ew = _graph(n, seed=70 + D)
    x = torch.from_numpy(np.random.default_rng(D).standard_normal((n, D)).astype(np.float32)).to(torch.float16)
    seeds = np.concatenate([np.arange(24), np.random.default_rng(2).integers(0, n, 150)]).astype(np.int32)
    _run(fsa, orc, indptr, indices, ew, x, seeds, fan, 6, "weighted fp16 D=%d fan=%s" % (D, fan), check_bwd=False)


def test_unit_weights_equal_the_unweighted_kernels(fsa):
    n, D = 3000, 128
    indptr, indices, _ = _graph(n, seed=9)
    dev = "cuda:0"
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    x = torch.randn((n, D), generator=torch.Generator().manual_seed(0)).to(dev)
    seeds = torch.from_numpy(np.random.default_rng(0).integers(0, n, 500).astype(np.int32)).to(dev)
    ones = torch.ones(indices.size, dtype=torch.float32, device=dev)
    for fan in ([12], [15, 10]):
        a = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, x, seeds, fan, 3)
        b = fsa.fsa_sample_wmean_fwd(d_indptr, d_indices, ones, x, seeds, fan, 3)
        assert torch.equal(a[2], b[2])
        assert torch.allclose(a[0], b[0], rtol=2e-6, atol=1e-6)
        if len(fan) == 2:
            assert torch.allclose(a[1], b[1], rtol=2e-6, atol=1e-6)


def test_weighted_large_shape_forward_backward(fsa, orc):
    """Product-graph shape at reduced size with hashed weights: a few thousand roots through
    the multi-tile-free fp32 path, forward + replay + backward."""
    from paper_2511_13645_amd import synth
    w = synth.make_workload("products", device="cuda:0", scale=0.05)
    g = w.graph
    ew = synth.hash_u01(11, 0, torch.arange(g.num_edges, device="cuda:0")).float()
    seeds = synth.seed_batches(g.num_nodes, 2048, 1, seed=2)[0]
    _run(fsa, orc, g.indptr.cpu().numpy(), g.indices.cpu().numpy(), ew.cpu().numpy(), w.x.cpu(), seeds.numpy(),
         [15, 10], 0, "weighted products@0.05")


@pytest.mark.parametrize("n_targets,B", [(3, 700), (100, 4096), (1000, 20000)])
def test_weighted_backward_with_heavily_shared_rows(fsa, orc, n_targets, B):
    """Every edge points into a small set of nodes, so the seeds of a workgroup keep hitting the
    same rows: the 1-hop weighted backward sums them in LDS (weight shares instead of 1/count),
    also with zero weights, seeds whose weights sum to zero and parallel edges."""
    rng = np.random.default_rng(n_targets)
    n, D, k = 30000, 96, 15
    deg = rng.integers(0, 40, size=n)
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    hot = rng.permutation(n)[:n_targets]
    p = 1.0 / np.arange(1, n_targets + 1) ** 1.2
    indices = hot[rng.choice(n_targets, size=int(indptr[-1]), p=p / p.sum())].astype(np.int32)
    ew = rng.random(indices.size).astype(np.float32)
    ew[rng.random(indices.size) < 0.1] = 0.0
    for v in range(0, n, 97):                                   # whole rows of zero weight
        ew[indptr[v]:indptr[v + 1]] = 0.0
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    seeds = np.concatenate([np.arange(0, n, 97)[:50], rng.integers(0, n, B - 50)]).astype(np.int32)
    _run(fsa, orc, indptr, indices, ew, x, seeds, [k], 3, "weighted shared rows %d" % n_targets)


def test_weighted_maximum_fanouts_with_one_wave_per_root(fsa, orc):
    """Fanouts 64/64 at a batch size that gives every root a single wave: the weighted strips
    (row offsets, weights, records for 4096 leaf slots) are the most LDS any launch asks for.
    The launch code sizes them against the device limit (more waves per root if one strip does
    not fit); the oracle checks the first 48 seeds, the backward runs over the whole batch."""
    n, D, B, fan = 3000, 32, 4100, [64, 64]
    indptr, indices, ew = _graph(n, seed=5, max_deg=200)
    rng = np.random.default_rng(0)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    seeds = rng.integers(0, n, B).astype(np.int32)
    dev = "cuda:0"
    r_out, r_h1, r_ids1, r_ids2, r_w1, r_w2 = orc.sample_wmean_fwd(indptr, indices, ew, x.numpy(), seeds[:48], fan, 3)
    d_x = x.to(dev)
    out, h1, ids1, ids2, w1, w2 = fsa.fsa_sample_wmean_fwd(torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev),
                                                           torch.from_numpy(ew).to(dev), d_x, torch.from_numpy(seeds).to(dev), fan, 3)
    torch.cuda.synchronize()
    assert_ids_equal(ids1[:48], r_ids1, "ids1")
    assert_ids_equal(ids2[:48], r_ids2, "ids2")
    assert np.array_equal(w1[:48].cpu().numpy(), r_w1) and np.array_equal(w2[:48].cpu().numpy(), r_w2)
    a_out, a_h1 = _scales(d_x, ids1[:48], ids2[:48], w1[:48], w2[:48])
    assert_close(to_f64(out[:48]), r_out, a_out, 1e-5, "out")
    assert_close(to_f64(h1[:48]), r_h1, a_h1, 1e-5, "out_h1")
    rp_out, rp_h1 = fsa.fsa_wmean_replay_fwd(d_x, ids1, w1, ids2, w2)
    torch.cuda.synchronize()
    assert torch.equal(rp_out, out) and torch.equal(rp_h1, h1)
    g = torch.from_numpy(rng.standard_normal((B, D)).astype(np.float32)).to(dev)
    gx = fsa.fsa_wmean_bwd(g, ids1, w1, ids2, w2, grad_x=torch.zeros((n, D), device=dev))
    torch.cuda.synchronize()
    a = (ids1.cpu().numpy(), w1.cpu().numpy(), ids2.cpu().numpy(), w2.cpu().numpy())
    want = orc.wmean_bwd(to_f64(g), *a, None, num_nodes=n)
    mag = orc.wmean_bwd(np.abs(to_f64(g)), *a, None, num_nodes=n)
    assert_close(to_f64(gx), want, mag, 1e-5, "grad_x")
