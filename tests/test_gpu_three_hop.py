"""GPU parity of the layer-wise two-hop forward and of the three-hop forward, replay and
backward against the CPU oracle: IDs and counts bit-exact, means within 1e-5 (fp32), 1e-2
(bf16) and 2e-3 (fp16: the three-hop `out` is formed from the rounded per-slot rows, two
half-ulp roundings of 2^-11 each), gradients within 1e-5.  Scales: the oracle's own nested
mean of |x| over the same IDs (every weight is positive), or its backward of |grad|."""
import numpy as np
import pytest
import torch

from parity_util import assert_close, assert_ids_equal, host_x, to_f64
from test_gpu_parity import ragged_graph

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL3 = {torch.float32: 1e-5, torch.bfloat16: 1e-2, torch.float16: 2e-3}


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _oracle_x(x):
    """(array, bf16 flag) the oracle takes for this table; fp16 is widened exactly."""
    if x.dtype == torch.float16:
        return x.to(torch.float64).numpy(), False
    return host_x(x)


def _dev_graph(indptr, indices):
    return torch.from_numpy(indptr).to(DEV), torch.from_numpy(indices).to(DEV)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_layerwise_two_hop(fsa, orc, dtype):
    n, D, B, fan = 4000, 96, 700, [15, 10]
    indptr, indices = ragged_graph(n, seed=3)
    rng = np.random.default_rng(4)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dtype)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    d_indptr, d_indices = _dev_graph(indptr, indices)
    d_x, d_seeds = x.to(DEV), torch.from_numpy(seeds).to(DEV)
    out, h1, m1, ids1, ids2 = fsa.fsa_sample_mean_layerwise_fwd(d_indptr, d_indices, d_x, d_seeds, fan, 9)
    o2, h2, i1, i2 = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, d_x, d_seeds, fan, 9)
    o1, _, j1, _ = fsa.fsa_sample_mean_fwd(d_indptr, d_indices, d_x, d_seeds, fan[:1], 9)
    torch.cuda.synchronize()
    u8 = lambda t: t.view(torch.uint8)
    assert torch.equal(u8(out), u8(o2)) and torch.equal(u8(h1), u8(h2)) and torch.equal(ids1, i1) and torch.equal(ids2, i2)
    assert torch.equal(u8(m1), u8(o1)) and torch.equal(ids1, j1)
    hx, is_bf16 = _oracle_x(x)
    r_m1, _, r_ids1, _ = orc.sample_mean_fwd(indptr, indices, hx, seeds, fan[:1], 9, bf16=is_bf16)
    a_m1, _, _, _ = orc.sample_mean_fwd(indptr, indices, np.abs(to_f64(x)), seeds, fan[:1], 9)
    assert_ids_equal(ids1, r_ids1, "ids1")
    assert_close(to_f64(m1), r_m1, a_m1, TOL3[dtype], "out_m1")


def three_hop_case(fsa, orc, indptr, indices, x, seeds, fan, seed, what, check_bwd=True, tol=None):
    n, D = x.shape
    B = len(seeds)
    tol = TOL3[x.dtype] if tol is None else tol
    hx, is_bf16 = _oracle_x(x)
    ref = orc.sample_mean3_fwd(indptr, indices, hx, seeds, fan, seed, bf16=is_bf16)
    d_indptr, d_indices = _dev_graph(indptr, indices)
    d_x, d_seeds = x.to(DEV), torch.from_numpy(seeds).to(DEV)
    r = fsa.fsa_sample_mean3_fwd(d_indptr, d_indices, d_x, d_seeds, fan, seed, emit_h2=True)
    torch.cuda.synchronize()
    for k in ("ids1", "ids2", "ids3", "cnt2"):
        assert_ids_equal(r[k], ref[k], what + " " + k)
    scale = orc.mean3_replay_fwd(np.abs(to_f64(x)), ref["ids1"], ref["ids2"], ref["ids3"])
    for k in ("out", "out_h1", "out_h2", "out_m1"):
        assert_close(to_f64(r[k]), ref[k], scale[k], tol, what + " " + k)

    # emission off: same means, bit for bit
    r0 = fsa.fsa_sample_mean3_fwd(d_indptr, d_indices, d_x, d_seeds, fan, seed, emit_h2=False, emit_ids=False)
    torch.cuda.synchronize()
    u8 = lambda t: t.view(torch.uint8)
    assert r0["ids2"] is None and r0["ids3"] is None and r0["out_h2"] is None
    for k in ("out", "out_h1", "out_m1"):
        assert torch.equal(u8(r0[k]), u8(r[k])), what + " emission-off " + k
    assert torch.equal(r0["cnt2"], r["cnt2"]) and torch.equal(r0["ids1"], r["ids1"])

    # replay: bitwise equal to the sampling forward
    rp = fsa.fsa_mean3_replay_fwd(d_x, r["ids1"], r["ids2"], r["ids3"], emit_h2=True)
    torch.cuda.synchronize()
    for k in ("out", "out_h1", "out_h2", "out_m1"):
        assert torch.equal(u8(rp[k]), u8(r[k])), what + " replay " + k
    assert torch.equal(rp["cnt2"], r["cnt2"])

    # replay with holes punched at every level
    rng = np.random.default_rng(12)
    ids1, ids2, ids3 = ref["ids1"].copy(), ref["ids2"].copy(), ref["ids3"].copy()
    ids3[rng.random(ids3.shape) < 0.3] = -1
    ids2[rng.random(ids2.shape) < 0.2] = -1
    ids1[rng.random(ids1.shape) < 0.2] = -1
    ref_h = orc.mean3_replay_fwd(hx, ids1, ids2, ids3, bf16=is_bf16)
    scale_h = orc.mean3_replay_fwd(np.abs(to_f64(x)), ids1, ids2, ids3)
    d_ids = [torch.from_numpy(a).to(DEV) for a in (ids1, ids2, ids3)]
    rh = fsa.fsa_mean3_replay_fwd(d_x, *d_ids, emit_h2=True)
    torch.cuda.synchronize()
    assert_ids_equal(rh["cnt2"], ref_h["cnt2"], what + " holes cnt2")
    for k in ("out", "out_h1", "out_h2", "out_m1"):
        assert_close(to_f64(rh[k]), ref_h[k], scale_h[k], tol, what + " holes " + k)

    if check_bwd and x.dtype == torch.float32:
        k1, k2, k3 = fan
        mk = lambda s, shape: torch.from_numpy(np.random.default_rng(s).standard_normal(shape).astype(np.float32)).to(DEV)
        G = {"out": mk(1, (B, D)), "h1": mk(2, (B, k1, D)), "h2": mk(3, (B, k1, k2, D)), "m1": mk(4, (B, D))}
        for use in ((), ("h1",), ("h2",), ("m1",), ("h1", "h2", "m1")):
            for ids_np, ids_dev, tag in (((ref["ids1"], ref["ids2"], ref["ids3"]), (r["ids1"], r["ids2"], r["ids3"]), "sampled"),
                                         ((ids1, ids2, ids3), d_ids, "holes")):
                kw = {"grad_" + k: G[k] for k in use}
                gx = torch.zeros((n, D), dtype=torch.float32, device=DEV)
                fsa.fsa_mean3_bwd(G["out"], *ids_dev, grad_x=gx, **kw)
                torch.cuda.synchronize()
                kw64 = {"grad_" + k: to_f64(G[k]) for k in use}
                want = orc.mean3_bwd(to_f64(G["out"]), *ids_np, num_nodes=n, **kw64)
                mag = orc.mean3_bwd(np.abs(to_f64(G["out"])), *ids_np, num_nodes=n,
                                    **{k: np.abs(v) for k, v in kw64.items()})
                assert_close(to_f64(gx), want, mag, 1e-5, "%s bwd %s %s" % (what, use, tag))
    return r


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("D", [64, 100, 301])
def test_three_hop_types_and_dims(fsa, orc, dtype, D):
    if dtype != torch.float32 and D == 301:
        D = 302
    n, B = 3000, 200
    indptr, indices = ragged_graph(n, seed=D, max_deg=40, hub_deg=900, wide=(D == 64))
    rng = np.random.default_rng(D)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dtype)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    three_hop_case(fsa, orc, indptr, indices, x, seeds, [15, 10, 5], 2**35 + D, "3-hop %s D=%d" % (dtype, D))


@pytest.mark.parametrize("fan", [[1, 1, 1], [3, 2, 64], [64, 1, 2], [2, 64, 3], [5, 5, 5], [7, 9, 11]])
def test_three_hop_fanout_range(fsa, orc, fan):
    n, D = 1500, 32
    B = 40 if max(fan) == 64 else 150
    indptr, indices = ragged_graph(n, seed=sum(fan), max_deg=80, hub_deg=700)
    rng = np.random.default_rng(sum(fan))
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32))
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    three_hop_case(fsa, orc, indptr, indices, x, seeds, fan, 17, "3-hop fan=%s" % fan)


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_three_hop_twenty_slots(fsa, orc, dtype):
    """k1 = 20 hop-1 slots per seed, B * k1 = 2400 roots of the inner launch."""
    n, D, B, fan = 2500, 72, 120, [20, 4, 3]
    indptr, indices = ragged_graph(n, seed=79, max_deg=50, hub_deg=600)
    rng = np.random.default_rng(80)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dtype)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    three_hop_case(fsa, orc, indptr, indices, x, seeds, fan, 5, "3-hop k1=20 %s" % dtype)


@pytest.mark.parametrize("D,dtype", [(602, torch.float32), (1024, torch.bfloat16), (1205, torch.float32)])
def test_three_hop_wide_rows(fsa, orc, D, dtype):
    """Rows of several 64-lane tiles (the multi-tile gather: 5 tiles, 2 tiles) and of more tiles
    than that gather takes (19 tiles of 4-byte chunks, walked tile by tile)."""
    n, B, fan = 1200, 60, [6, 5, 4]
    indptr, indices = ragged_graph(n, seed=D, max_deg=30, hub_deg=300)
    rng = np.random.default_rng(D)
    x = torch.from_numpy(rng.standard_normal((n, D)).astype(np.float32)).to(dtype)
    seeds = np.concatenate([np.arange(8), rng.integers(0, n, B - 8)]).astype(np.int32)
    three_hop_case(fsa, orc, indptr, indices, x, seeds, fan, 21, "3-hop D=%d" % D)


def test_three_hop_empty_batch_and_degenerate_graph(fsa, orc):
    n, D = 50, 16
    indptr = np.zeros(n + 1, dtype=np.int32)                     # no edges at all
    indices = np.zeros(0, dtype=np.int32)
    x = torch.randn((n, D))
    seeds = np.arange(10, dtype=np.int32)
    d_indptr, d_indices = _dev_graph(indptr, np.zeros(1, dtype=np.int32))
    r = fsa.fsa_sample_mean3_fwd(d_indptr, d_indices, x.to(DEV), torch.from_numpy(seeds).to(DEV), [4, 3, 2], 1, emit_h2=True)
    torch.cuda.synchronize()
    assert (r["out"] == 0).all() and (r["out_h1"] == 0).all() and (r["out_h2"] == 0).all() and (r["out_m1"] == 0).all()
    assert (r["ids1"] == -1).all() and (r["ids2"] == -1).all() and (r["ids3"] == -1).all() and (r["cnt2"] == 0).all()
    gx = torch.zeros((n, D), device=DEV)
    fsa.fsa_mean3_bwd(torch.ones((10, D), device=DEV), r["ids1"], r["ids2"], r["ids3"], grad_x=gx)
    torch.cuda.synchronize()
    assert (gx == 0).all()
    e = torch.zeros(0, dtype=torch.int32, device=DEV)
    r = fsa.fsa_sample_mean3_fwd(d_indptr, d_indices, x.to(DEV), e, [4, 3, 2], 1)
    assert r["out"].shape == (0, D)
