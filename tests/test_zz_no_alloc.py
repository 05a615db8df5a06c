"""fsa_mean3_bwd_noalloc (the three-hop backward on the library's fixed scratch array, for
callers that cannot allocate) against fsa_mean3_bwd with a caller workspace: two calls in a
row through the C ABI, the second on a smaller input, each within the backward's tolerance of
the workspace variant; sizes beyond the fixed array are refused."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(n, D, B, fan, seed, dev):
    from paper_2511_13645_amd import binding
    rng = np.random.default_rng(seed)
    deg = rng.integers(0, 40, n)
    deg[:4] = [0, 1, 500, 39]
    indptr = torch.from_numpy(np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)).to(dev)
    indices = torch.from_numpy(rng.integers(0, n, int(deg.sum())).astype(np.int32)).to(dev)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dev)
    seeds = torch.from_numpy(rng.integers(0, n, B).astype(np.int32)).to(dev)
    r = binding.fsa_sample_mean3_fwd(indptr, indices, x, seeds, fan, 5)
    k1, k2, k3 = fan
    g = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float32)).to(dev)
    return dict(ids1=r["ids1"], ids2=r["ids2"], ids3=r["ids3"], go=g(B, D), g1=g(B, k1, D), g2=g(B, k1, k2, D), gm=g(B, D),
                n=n, D=D, B=B, fan=fan)


def _both(L, c, dev):
    """grad_x by the workspace variant, by the no-alloc variant, and the sum of |contributions|."""
    st = torch.cuda.current_stream().cuda_stream
    k1, k2, k3 = c["fan"]
    P = lambda t: t.data_ptr()
    outs = []
    for mode in ("work", "noalloc", "scale"):
        gx = torch.zeros((c["n"], c["D"]), device=dev)
        go, g1, g2, gm = (c[k].abs() if mode == "scale" else c[k] for k in ("go", "g1", "g2", "gm"))
        if mode == "noalloc":
            rc = L.fsa_mean3_bwd_noalloc(P(go), P(g1), P(g2), P(gm), P(c["ids1"]), P(c["ids2"]), P(c["ids3"]),
                                         c["B"], k1, k2, k3, c["D"], P(gx), c["n"], st)
        else:
            work = torch.empty((c["B"], k1, c["D"]), device=dev)
            rc = L.fsa_mean3_bwd(P(go), P(g1), P(g2), P(gm), P(c["ids1"]), P(c["ids2"]), P(c["ids3"]),
                                 c["B"], k1, k2, k3, c["D"], P(gx), c["n"], P(work), st)
        assert rc == 0, (mode, rc)
        torch.cuda.synchronize()
        outs.append(gx.double().cpu().numpy())
    return outs


def test_noalloc_three_hop_backward_matches_the_workspace_variant_twice_in_a_row():
    from paper_2511_13645_amd import binding
    L = binding.lib()
    dev = "cuda:0"
    big = _case(6000, 96, 900, (7, 5, 4), 1, dev)
    small = _case(800, 33, 50, (3, 2, 6), 2, dev)            # second call: smaller in every dimension
    for name, c in (("first call", big), ("second, smaller call", small), ("third call, large again", big)):
        ref, got, scale = _both(L, c, dev)
        bound = 1e-5 * np.maximum(np.abs(ref), scale)          # the backward's bar: 1e-5 * sum |contribution|
        err = np.abs(got - ref)
        assert np.isfinite(got).all() and (err <= bound).all(), "%s: max excess %g" % (name, (err - bound).max())
        assert np.abs(ref).max() > 0
    # beyond the fixed array: refused before anything is launched, grad_x untouched
    k1, k2, k3 = 64, 1, 1
    B, D = binding.FSA_SCRATCH_FLOATS // (k1 * 512) + 1, 512
    gx = torch.zeros((16, D), device=dev)
    z = torch.zeros(8, device=dev)
    zi = torch.zeros(8, dtype=torch.int32, device=dev)
    rc = L.fsa_mean3_bwd_noalloc(z.data_ptr(), None, None, None, zi.data_ptr(), zi.data_ptr(), zi.data_ptr(),
                                 B, k1, k2, k3, D, gx.data_ptr(), 16, torch.cuda.current_stream().cuda_stream)
    assert rc == -6 and "scratch" in binding.status_string(rc)
    torch.cuda.synchronize()
    assert float(gx.abs().sum()) == 0.0
