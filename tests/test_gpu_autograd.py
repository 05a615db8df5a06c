"""The autograd wrapper: gradients through the fused operator equal the oracle's backward,
and a training step moves a learnable table only where rows were sampled."""
import numpy as np
import pytest
import torch

from parity_util import assert_close, to_f64

pytestmark = pytest.mark.gpu


def _graph(n, seed):
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, 60, size=n)
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    indices = rng.integers(0, n, size=int(indptr[-1])).astype(np.int32)
    return indptr, indices


@pytest.mark.parametrize("fan", [[10], [6, 5]])
def test_autograd_matches_oracle_backward(orc, fan):
    from paper_2511_13645_amd.autograd import fused_sample_mean
    dev = "cuda:0"
    n, D, B = 2000, 40, 300
    indptr, indices = _graph(n, 1)
    rng = np.random.default_rng(2)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dev).requires_grad_(True)
    seeds = torch.from_numpy(rng.integers(0, n, B).astype(np.int32)).to(dev)
    out, h1, ids1, ids2 = fused_sample_mean(x, torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev),
                                            seeds, fan, 11, want_h1=True)
    w_out = torch.from_numpy(rng.standard_normal(out.shape).astype(np.float32)).to(dev)
    loss = (out * w_out).sum()
    w_h1 = None
    if len(fan) == 2:
        w_h1 = torch.from_numpy(rng.standard_normal(h1.shape).astype(np.float32)).to(dev)
        loss = loss + (h1 * w_h1).sum()
    loss.backward()
    torch.cuda.synchronize()
    r_out, r_h1, r_ids1, r_ids2 = orc.sample_mean_fwd(indptr, indices, x.detach().cpu().numpy(), seeds.cpu().numpy(), fan, 11)
    assert np.array_equal(ids1.cpu().numpy(), r_ids1)
    r_gx = orc.mean_bwd(to_f64(w_out), r_ids1, r_ids2, None if w_h1 is None else to_f64(w_h1), num_nodes=n)
    scale = orc.mean_bwd(np.abs(to_f64(w_out)), r_ids1, r_ids2, None if w_h1 is None else np.abs(to_f64(w_h1)), num_nodes=n)
    assert_close(to_f64(x.grad), r_gx, scale, 1e-5, "autograd grad_x fan=%s" % fan)


def test_no_ids_without_grad_and_training_step_touches_sampled_rows_only():
    from paper_2511_13645_amd.autograd import fused_sample_mean
    dev = "cuda:0"
    n, D, B = 3000, 32, 128
    indptr, indices = _graph(n, 3)
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    seeds = torch.arange(B, dtype=torch.int32, device=dev)
    x_fixed = torch.randn((n, D), device=dev)
    out, h1, ids1, ids2 = fused_sample_mean(x_fixed, d_indptr, d_indices, seeds, [5, 4], 0)
    assert ids1 is None and ids2 is None and h1 is None           # nothing saved, nothing emitted
    table = torch.nn.Parameter(x_fixed.clone())
    opt = torch.optim.SGD([table], lr=0.5)
    out, _, ids1, ids2 = fused_sample_mean(table, d_indptr, d_indices, seeds, [5, 4], 0)
    out.square().sum().backward()
    opt.step()
    torch.cuda.synchronize()
    moved = (table.detach() != x_fixed).any(dim=1)
    sampled = torch.zeros(n, dtype=torch.bool, device=dev)
    sampled[ids2[ids2 >= 0].long()] = True
    assert not (moved & ~sampled).any()
    assert moved.sum() > 0.5 * sampled.sum()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("fan,D", [([10], 40), ([6, 5], 40), ([6, 5], 33)])
def test_autograd_with_16bit_tables(orc, dtype, fan, D):
    """A 16-bit table gets a gradient of its own type (packed atomics; an odd D goes through an
    fp32 master and is rounded once), or the caller's fp32 master gradient is accumulated into."""
    from paper_2511_13645_amd.autograd import fused_sample_mean
    dev = "cuda:0"
    n, B = 2000, 300
    ulp = {torch.bfloat16: 2.0 ** -8, torch.float16: 2.0 ** -10}[dtype]
    indptr, indices = _graph(n, 1)
    d_indptr, d_indices = torch.from_numpy(indptr).to(dev), torch.from_numpy(indices).to(dev)
    rng = np.random.default_rng(2)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dev).to(dtype).requires_grad_(True)
    seeds = torch.from_numpy(rng.integers(0, n, B).astype(np.int32)).to(dev)
    w_out = torch.from_numpy(rng.standard_normal((B, D)).astype(np.float32)).to(dev).to(dtype)

    out, _, ids1, ids2 = fused_sample_mean(x, d_indptr, d_indices, seeds, fan, 11)
    (out * w_out).sum().backward()
    torch.cuda.synchronize()
    assert x.grad.dtype == dtype
    h1 = ids1.cpu().numpy()
    h2 = None if ids2 is None else ids2.cpu().numpy()
    ref = orc.mean_bwd(to_f64(w_out), h1, h2, None, num_nodes=n)
    mag = orc.mean_bwd(np.abs(to_f64(w_out)), h1, h2, None, num_nodes=n)
    leaves = h1 if h2 is None else h2
    n_add = np.bincount(leaves[leaves >= 0], minlength=n).astype(np.float64)[:, None]
    err = np.abs(to_f64(x.grad) - ref)
    assert (err <= (n_add + 1) * (ulp * mag + 2.0 ** -24)).all()

    master = torch.zeros((n, D), dtype=torch.float32, device=dev)
    x2 = x.detach().clone().requires_grad_(True)
    out2, _, _, _ = fused_sample_mean(x2, d_indptr, d_indices, seeds, fan, 11, master_grad=master)
    (out2 * w_out).sum().backward()
    torch.cuda.synchronize()
    assert x2.grad is None
    assert_close(to_f64(master), ref, mag, 1e-5, "master gradient %s fan=%s" % (dtype, fan))
