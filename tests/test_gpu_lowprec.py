"""GPU parity of the reduced-precision path (the paper lists FP32-only kernels as a limitation,
Sec. 5): fp16 feature tables in the forward and replay, and the backward with 16-bit upstream
gradients into an fp32 master gradient or into a 16-bit grad_x by packed atomics.

The oracle needs no arithmetic of its own for this: every 16-bit input converts to fp64
exactly, the oracle computes in fp64, and the bound on the difference comes from the rounding
steps the HIP path is documented to take:
  forward, fp16 out      fp32 accumulation (as for fp32 tables) + one rounding to fp16,
                         half an ulp = 2^-11 relative  ->  tolerance 1e-3;
  backward, fp32 grad_x  nothing is rounded below fp32  ->  the fp32 tolerance 1e-5;
  backward, 16-bit grad_x  each contribution is rounded once and each of the n atomic adds
                         into an element rounds the running sum, at most one ulp each whatever
                         the rounding mode: |error| <= (n + 1) * ulp * sum|contribution|, with
                         ulp = 2^-8 (bf16) or 2^-10 (fp16); n is counted from the IDs.  Below the
                         smallest normal number a rounding is absolute, not relative: each of
                         the n + 1 roundings may also cost one subnormal spacing (2^-24 for fp16,
                         2^-133 for bf16)."""
import numpy as np
import pytest
import torch

from parity_util import assert_close, assert_ids_equal, forward_scales, to_f64
from test_gpu_parity import ragged_graph

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ULP = {torch.bfloat16: 2.0 ** -8, torch.float16: 2.0 ** -10}
SUBNORMAL_STEP = {torch.bfloat16: 2.0 ** -133, torch.float16: 2.0 ** -24}


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


@pytest.mark.parametrize("D", [1, 2, 6, 64, 100, 128, 301, 1024])
@pytest.mark.parametrize("fan", [[15], [15, 10]])
def test_fp16_features_forward_and_replay(fsa, orc, D, fan):
    n, B = 3000, 517
    indptr, indices = ragged_graph(n, seed=D, wide=(D % 2 == 0))
    rng = np.random.default_rng(D + 1)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(torch.float16)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    seed = 77 + D
    x64 = x.to(torch.float64).numpy()                       # exact
    r_out, r_h1, r_ids1, r_ids2 = orc.sample_mean_fwd(indptr, indices, x64, seeds, fan, seed)

    d_x = x.to(DEV)
    out, h1, ids1, ids2 = fsa.fsa_sample_mean_fwd(torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV),
                                                  d_x, torch.from_numpy(seeds).to(DEV), fan, seed)
    torch.cuda.synchronize()
    assert out.dtype == torch.float16
    assert_ids_equal(ids1, r_ids1, "ids1")
    if len(fan) == 2:
        assert_ids_equal(ids2, r_ids2, "ids2")
    a_out, a_h1 = forward_scales(d_x, ids1, ids2)
    assert_close(to_f64(out), r_out, a_out, 1e-3, "fp16 out")
    if len(fan) == 2:
        assert_close(to_f64(h1), r_h1, a_h1, 1e-3, "fp16 out_h1")
    rp_out, rp_h1 = fsa.fsa_mean_replay_fwd(d_x, ids1, ids2)
    torch.cuda.synchronize()
    assert torch.equal(rp_out.view(torch.int16), out.view(torch.int16))
    if len(fan) == 2:
        assert torch.equal(rp_h1.view(torch.int16), h1.view(torch.int16))


def adds_per_row(ids1: np.ndarray, ids2, n: int) -> np.ndarray:
    """Upper bound on the number of atomic additions each row of grad_x receives: one per
    (slot, distinct ID in the slot)."""
    ids = ids1[:, None, :] if ids2 is None else ids2
    flat = ids.reshape(-1, ids.shape[-1])
    s = np.sort(flat, axis=1)
    first = np.ones_like(s, dtype=bool)
    first[:, 1:] = s[:, 1:] != s[:, :-1]
    keep = first & (s >= 0)
    return np.bincount(s[keep], minlength=n)


def lowprec_case(fsa, orc, indptr, indices, n, D, seeds, fan, g_dtype, x_dtype, what):
    rng = np.random.default_rng(11)
    xf = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(DEV)
    d_seeds = torch.from_numpy(seeds).to(DEV)
    _, _, ids1, ids2 = fsa.fsa_sample_mean_fwd(torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV),
                                               xf, d_seeds, fan, 5, emit_h1=False)
    B = len(seeds)
    g = torch.from_numpy(np.random.default_rng(3).standard_normal((B, D)).astype(np.float32)).to(DEV).to(g_dtype)
    gh = None
    if len(fan) == 2:
        gh = torch.from_numpy(np.random.default_rng(4).standard_normal((B, fan[0], D)).astype(np.float32)).to(DEV).to(g_dtype)
    gx = torch.zeros((n, D), dtype=x_dtype, device=DEV)
    fsa.fsa_mean_bwd_lp(g, ids1, ids2, gh, grad_x=gx)
    torch.cuda.synchronize()
    h_ids1 = ids1.cpu().numpy()
    h_ids2 = None if ids2 is None else ids2.cpu().numpy()
    g64, gh64 = to_f64(g), None if gh is None else to_f64(gh)          # exact widenings
    ref = orc.mean_bwd(g64, h_ids1, h_ids2, gh64, num_nodes=n)
    mag = orc.mean_bwd(np.abs(g64), h_ids1, h_ids2, None if gh64 is None else np.abs(gh64), num_nodes=n)
    if x_dtype == torch.float32:
        assert_close(to_f64(gx), ref, mag, 1e-5, what)
    else:
        n_add = adds_per_row(h_ids1, h_ids2, n).astype(np.float64)[:, None]
        got = to_f64(gx)
        assert np.isfinite(got).all(), what
        bound = (n_add + 1.0) * (ULP[x_dtype] * mag + SUBNORMAL_STEP[x_dtype])
        err = np.abs(got - ref)
        assert (err <= bound).all(), "%s: worst excess %g at %s" % (
            what, float((err - bound).max()), np.unravel_index(np.argmax(err - bound), err.shape))
        # the bound is not vacuous: rows that took a single addition are within one rounding
        once = n_add[:, 0] == 1
        if once.any():
            assert (err[once] <= 2.0 * (ULP[x_dtype] * mag[once] + SUBNORMAL_STEP[x_dtype])).all(), what + " single-add rows"
        # and rows that took none are untouched
        assert (got[n_add[:, 0] == 0] == 0).all(), what + " untouched rows"


COMBOS = [(torch.float32, torch.float32), (torch.bfloat16, torch.float32), (torch.float16, torch.float32),
          (torch.float32, torch.bfloat16), (torch.bfloat16, torch.bfloat16),
          (torch.float32, torch.float16), (torch.float16, torch.float16)]


@pytest.mark.parametrize("g_dtype,x_dtype", COMBOS)
@pytest.mark.parametrize("fan", [[15], [15, 10]])
def test_backward_types(fsa, orc, g_dtype, x_dtype, fan):
    # an fp32 grad_x takes any D; a 16-bit one is added to in element pairs
    for D in (2, 64, 100, 602) + ((7, 301) if x_dtype == torch.float32 else ()):
        n = 2500
        indptr, indices = ragged_graph(n, seed=D + len(fan))
        rng = np.random.default_rng(D)
        B = 300 if len(fan) == 2 else 900
        seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
        lowprec_case(fsa, orc, indptr, indices, n, D, seeds, fan, g_dtype, x_dtype,
                     "bwd %s -> %s D=%d fan=%s" % (g_dtype, x_dtype, D, fan))


@pytest.mark.parametrize("x_dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_backward_types_with_shared_rows(fsa, orc, x_dtype):
    """Rows shared by many seeds of a workgroup go through the in-LDS (fp32) aggregation of the
    1-hop backward before they reach the 16-bit table."""
    rng = np.random.default_rng(5)
    n, D, k, B = 20000, 96, 15, 6000
    deg = rng.integers(0, 40, size=n)
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    hot = rng.permutation(n)[:50]
    p = 1.0 / np.arange(1, 51) ** 1.2
    indices = hot[rng.choice(50, size=int(indptr[-1]), p=p / p.sum())].astype(np.int32)
    seeds = rng.integers(0, n, B).astype(np.int32)
    g_dtype = torch.float32 if x_dtype == torch.float32 else x_dtype
    lowprec_case(fsa, orc, indptr, indices, n, D, seeds, [k], g_dtype, x_dtype, "shared rows -> %s" % x_dtype)


def test_fp32_pair_is_the_plain_backward(fsa):
    """grad_dtype == grad_x_dtype == fp32 runs the same kernels as fsa_mean_bwd."""
    n, D, B = 2000, 64, 512
    indptr, indices = ragged_graph(n, seed=1)
    rng = np.random.default_rng(0)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(DEV)
    seeds = torch.from_numpy(rng.permutation(n)[:B].astype(np.int32)).to(DEV)
    _, _, ids1, _ = fsa.fsa_sample_mean_fwd(torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV),
                                            x, seeds, [15], 1)
    # distinct rows per seed and distinct seeds do not make the adds of two runs commute in
    # general, so compare to tolerance only
    g = torch.from_numpy(rng.standard_normal((B, D)).astype(np.float32)).to(DEV)
    a = fsa.fsa_mean_bwd(g, ids1, grad_x=torch.zeros((n, D), device=DEV))
    b = fsa.fsa_mean_bwd_lp(g, ids1, grad_x=torch.zeros((n, D), device=DEV))
    torch.cuda.synchronize()
    assert torch.allclose(a, b, rtol=1e-5, atol=1e-6)
