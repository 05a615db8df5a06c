"""The Python binding refuses mismatched shapes, types and devices before the C call: a wrong
shape would otherwise become an out-of-bounds store or atomic on the device."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def case(fsa):
    dev = "cuda:0"
    rng = np.random.default_rng(0)
    n, D, B, k1, k2 = 200, 16, 12, 5, 4
    deg = rng.integers(0, 12, n)
    indptr = torch.from_numpy(np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)).to(dev)
    indices = torch.from_numpy(rng.integers(0, n, int(deg.sum())).astype(np.int32)).to(dev)
    x = torch.randn((n, D), device=dev)
    seeds = torch.from_numpy(rng.integers(0, n, B).astype(np.int32)).to(dev)
    out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(indptr, indices, x, seeds, [k1, k2], 1)
    ew = torch.rand(indices.shape[0], device=dev)
    _, _, _, _, w1, w2 = fsa.fsa_sample_wmean_fwd(indptr, indices, ew, x, seeds, [k1, k2], 1)
    torch.cuda.synchronize()
    return dict(n=n, D=D, B=B, k1=k1, k2=k2, indptr=indptr, indices=indices, x=x, seeds=seeds, ids1=ids1, ids2=ids2,
                w1=w1, w2=w2, ew=ew, dev=dev)


def test_forward_and_replay_refuse_wrong_outputs(fsa, case):
    c = case
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device=c["dev"])
    with pytest.raises(ValueError):
        fsa.fsa_sample_mean_fwd(c["indptr"], c["indices"], c["x"], c["seeds"], [c["k1"], c["k2"]], 1, out=z(c["B"] - 1, c["D"]))
    with pytest.raises(ValueError):
        fsa.fsa_sample_mean_fwd(c["indptr"], c["indices"], c["x"], c["seeds"], [c["k1"], c["k2"]], 1,
                                out_ids2=z(c["B"], c["k1"], c["k2"] - 1, dt=torch.int32))
    with pytest.raises(TypeError):
        fsa.fsa_sample_mean_fwd(c["indptr"], c["indices"], c["x"], c["seeds"], [c["k1"]], 1, out=z(c["B"], c["D"], dt=torch.bfloat16))
    with pytest.raises(ValueError):
        fsa.fsa_sample_mean_fwd(c["indptr"][:-1], c["indices"], c["x"], c["seeds"], [c["k1"]], 1)
    with pytest.raises(ValueError):
        fsa.fsa_mean_replay_fwd(c["x"], c["ids1"], c["ids2"], out=z(c["B"], c["D"] + 1))
    with pytest.raises(ValueError):
        fsa.fsa_mean_replay_fwd(c["x"], c["ids1"], c["ids2"], out_h1=z(c["B"], c["k1"] + 1, c["D"]))
    with pytest.raises(ValueError):
        fsa.fsa_mean_replay_fwd(c["x"], c["ids1"], c["ids2"][:-1])
    with pytest.raises(ValueError):
        fsa.fsa_mean_replay_fwd(c["x"], c["ids1"], c["ids2"], out=torch.zeros((c["B"], c["D"])))       # host tensor


def test_backward_wrappers_refuse_wrong_shapes(fsa, case):
    c = case
    B, D, n, k1, k2 = c["B"], c["D"], c["n"], c["k1"], c["k2"]
    z = lambda *s: torch.zeros(s, device=c["dev"])
    g, gx = z(B, D), z(n, D)
    for bad in (dict(grad_out=z(B + 1, D)), dict(grad_x=z(n, D + 1)), dict(ids2=c["ids2"][:, :-1]),
                dict(grad_h1=z(B, k1, D + 1)), dict(ids2=c["ids2"][:-1])):
        a = dict(grad_out=g, ids1=c["ids1"], ids2=c["ids2"], grad_h1=None, grad_x=gx)
        a.update(bad)
        for fn in (fsa.fsa_mean_bwd, fsa.fsa_mean_bwd_lp):
            with pytest.raises(ValueError):
                fn(a["grad_out"], a["ids1"], a["ids2"].contiguous(), a["grad_h1"], grad_x=a["grad_x"])
    for bad in (dict(grad_out=z(B + 1, D)), dict(grad_x=z(n, D + 1)), dict(w1=c["w1"][:-1]), dict(w2=c["w2"][:, :, :-1]),
                dict(grad_h1=z(B, k1 - 1, D)), dict(w2=None)):
        a = dict(grad_out=g, ids1=c["ids1"], w1=c["w1"], ids2=c["ids2"], w2=c["w2"], grad_h1=None, grad_x=gx)
        a.update(bad)
        with pytest.raises(ValueError):
            fsa.fsa_wmean_bwd(a["grad_out"], a["ids1"], a["w1"].contiguous(), a["ids2"],
                              None if a["w2"] is None else a["w2"].contiguous(), a["grad_h1"], grad_x=a["grad_x"])
    with pytest.raises(ValueError):
        fsa.fsa_wmean_replay_fwd(c["x"], c["ids1"], c["w1"][:-1].contiguous(), c["ids2"], c["w2"])
    with pytest.raises(ValueError):
        fsa.fsa_wmean_replay_fwd(c["x"], c["ids1"], c["w1"], c["ids2"], c["w2"][:, :-1].contiguous())
    # three-hop backward
    ids3 = torch.full((B, k1, k2, 3), -1, dtype=torch.int32, device=c["dev"])
    with pytest.raises(ValueError):
        fsa.fsa_mean3_bwd(z(B + 1, D), c["ids1"], c["ids2"], ids3, grad_x=gx)
    with pytest.raises(ValueError):
        fsa.fsa_mean3_bwd(g, c["ids1"], c["ids2"], ids3, grad_x=z(n, D + 2))
    with pytest.raises(ValueError):
        fsa.fsa_mean3_bwd(g, c["ids1"][:-1], c["ids2"], ids3, grad_x=gx)
    # nothing above may have touched grad_x
    torch.cuda.synchronize()
    assert float(gx.abs().sum()) == 0.0
