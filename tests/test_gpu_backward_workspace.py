"""fsa_mean_bwd_ws: the 2-hop backward that owns every destination row (bins by row, sorts in
LDS, one plain update per distinct row) against the oracle's backward and against the atomic
backward, on wide-row shapes and large batches of narrower rows that take that route and on
shapes that must fall back."""
import numpy as np
import pytest
import torch

from parity_util import assert_close, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fsa():
    from paper_2511_13645_amd import binding
    binding.lib()
    return binding


def _ids(rng, B, k1, k2, n, holes=0.1, dup=True, targets=None):
    """Saved-ID arrays with holes anywhere, empty slots, parallel edges, shared rows."""
    pick = (lambda size: rng.integers(0, n, size)) if targets is None else (lambda size: targets[rng.integers(0, len(targets), size)])
    ids1 = pick((B, k1)).astype(np.int32)
    ids2 = pick((B, k1, k2)).astype(np.int32)
    ids2[rng.random((B, k1, k2)) < holes] = -1
    ids1[rng.random((B, k1)) < holes] = -1
    ids2[ids1 < 0] = -1
    if dup and k2 > 1:
        ids2[:, :, 1] = np.where(ids2[:, :, 0] >= 0, ids2[:, :, 0], ids2[:, :, 1])     # the same row twice in a slot
    ids2[::7, 0, :] = -1                                                                # slots without rows
    if B > 3:
        ids2[3] = -1                                                                    # a root with nothing
    return ids1, ids2


def _check(fsa, orc, B, k1, k2, D, n, seed, with_h1=True, targets=None, expect_route=True, reproducible=True):
    rng = np.random.default_rng(seed)
    dev = "cuda:0"
    ids1, ids2 = _ids(rng, B, k1, k2, n, targets=targets)
    g = rng.standard_normal((B, D)).astype(np.float32)
    gh = rng.standard_normal((B, k1, D)).astype(np.float32) if with_h1 else None
    need = fsa.fsa_mean_bwd_workspace_bytes(B, k1, k2, D)
    assert (need > 0) == expect_route, (need, expect_route)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    d = dict(g=torch.from_numpy(g).to(dev), gh=None if gh is None else torch.from_numpy(gh).to(dev),
             i1=torch.from_numpy(ids1).to(dev), i2=torch.from_numpy(ids2).to(dev))
    base = rng.standard_normal((n, D)).astype(np.float32)               # grad_x is accumulated into
    gx = torch.from_numpy(base.copy()).to(dev)
    fsa.fsa_mean_bwd_ws(d["g"], d["i1"], d["i2"], d["gh"], grad_x=gx, workspace=ws)
    fsa.fsa_mean_bwd_ws(d["g"], d["i1"], d["i2"], d["gh"], grad_x=gx, workspace=ws)      # twice: the workspace is reusable
    gx_at = torch.from_numpy(base.copy()).to(dev)
    fsa.fsa_mean_bwd(d["g"], d["i1"], d["i2"], d["gh"], grad_x=gx_at)
    torch.cuda.synchronize()
    ref = orc.mean_bwd(g.astype(np.float64), ids1, ids2, None if gh is None else gh.astype(np.float64), num_nodes=n)
    mag = orc.mean_bwd(np.abs(g).astype(np.float64), ids1, ids2, None if gh is None else np.abs(gh).astype(np.float64), num_nodes=n)
    assert_close(to_f64(gx) - base, 2 * ref, 2 * mag + 1e-6 * np.abs(base) / 1e-5, 1e-5, "grad_x (workspace route)")
    assert_close(to_f64(gx_at) - base, ref, mag + 1e-6 * np.abs(base) / 1e-5, 1e-5, "grad_x (atomic route)")
    if expect_route:
        # the owning route is bit-reproducible when no bin overflows
        gx2 = torch.from_numpy(base.copy()).to(dev)
        fsa.fsa_mean_bwd_ws(d["g"], d["i1"], d["i2"], d["gh"], grad_x=gx2, workspace=ws)
        gx3 = torch.from_numpy(base.copy()).to(dev)
        fsa.fsa_mean_bwd_ws(d["g"], d["i1"], d["i2"], d["gh"], grad_x=gx3, workspace=ws)
        torch.cuda.synchronize()
        if targets is None and reproducible:
            assert torch.equal(gx2, gx3), "two runs of the owning route differ"


@pytest.mark.parametrize("D", [256, 260, 602, 1000, 513, 2048])
def test_wide_rows_take_the_owning_route(fsa, orc, D):
    # D=256: 16-byte chunks, one tile; 260: 16-byte, two tiles; 602 / 1000: 8-byte chunks, 5 / 8 tiles (1000 = 16-byte, 4);
    # 513: 4-byte chunks would need 9 tiles -> falls back inside the call although the shape is eligible; 2048: 16-byte, 8 tiles
    B, k1, k2 = 256, 7, 10
    while B * k1 * k2 * D * 4 < (36 << 20):
        B *= 2
    _check(fsa, orc, B, k1, k2, D, 20000, D, with_h1=(D != 1000), reproducible=(D != 513))


def test_social_like_shape_with_shared_rows(fsa, orc):
    """Fanouts 25/10, D=602: leaves drawn from a power-law over few nodes, so many rows are hit by several roots."""
    rng = np.random.default_rng(1)
    n = 30000
    p = 1.0 / np.arange(1, n + 1) ** 0.8
    targets = rng.choice(n, size=200000, p=p / p.sum()).astype(np.int32)
    _check(fsa, orc, 700, 25, 10, 602, n, 11, targets=targets)


def test_a_hub_overflows_its_bin(fsa, orc):
    """Every leaf is one of three rows: their bins overflow, the overflow entries and the bins' own sums go in by atomics."""
    targets = np.array([5, 77, 1234], dtype=np.int32)
    _check(fsa, orc, 600, 20, 10, 300, 2000, 3, targets=targets)


@pytest.mark.parametrize("D", [64, 100, 128, 130, 200, 255])
def test_large_batches_of_narrow_rows_take_the_owning_route(fsa, orc, D):
    # rows of 256 .. 1020 bytes: groups of 16 / 32 / 64 lanes per row (D=64: 16 chunks of 16 bytes; 100: 25; 128: 32;
    # 130: 65 chunks of 8 bytes, more than one wave's lanes -> the wide-row kernel; 200: 50; 255: 4-byte chunks -> wide-row kernel)
    B, k1, k2 = 4096, 10, 10                                       # 409,600 leaf slots
    _check(fsa, orc, B, k1, k2, D, 50000, D, with_h1=(D != 200))


def test_narrow_rows_with_a_hub_overflowing_its_bin(fsa, orc):
    targets = np.concatenate([np.full(3000, 9, dtype=np.int32), np.arange(100, 20000, dtype=np.int32)])
    _check(fsa, orc, 4096, 10, 10, 96, 20000, 4, targets=targets)


@pytest.mark.parametrize("shape", [(64, 5, 4, 602), (1024, 15, 10, 100), (8192, 10, 10, 48), (512, 10, 0, 602)])
def test_small_narrow_and_one_hop_calls_fall_back_to_atomics(fsa, orc, shape):
    B, k1, k2, D = shape
    if k2 == 0:                                                    # 1-hop
        rng = np.random.default_rng(0)
        dev = "cuda:0"
        n = 5000
        ids1 = rng.integers(-1, n, (B, k1)).astype(np.int32)
        g = rng.standard_normal((B, D)).astype(np.float32)
        ws = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
        gx = torch.zeros((n, D), device=dev)
        fsa.fsa_mean_bwd_ws(torch.from_numpy(g).to(dev), torch.from_numpy(ids1).to(dev), grad_x=gx, workspace=ws)
        torch.cuda.synchronize()
        ref = orc.mean_bwd(g.astype(np.float64), ids1, num_nodes=n)
        mag = orc.mean_bwd(np.abs(g).astype(np.float64), ids1, num_nodes=n)
        assert_close(to_f64(gx), ref, mag, 1e-5, "1-hop through the workspace entry point")
        return
    _check(fsa, orc, B, k1, k2, D, 8000, 5, expect_route=False)


def test_missing_small_or_misaligned_workspace_falls_back(fsa, orc):
    rng = np.random.default_rng(2)
    dev = "cuda:0"
    B, k1, k2, D, n = 1024, 10, 10, 512, 10000
    ids1, ids2 = _ids(rng, B, k1, k2, n)
    g = rng.standard_normal((B, D)).astype(np.float32)
    need = fsa.fsa_mean_bwd_workspace_bytes(B, k1, k2, D)
    assert need > 0
    ref = orc.mean_bwd(g.astype(np.float64), ids1, ids2, num_nodes=n)
    mag = orc.mean_bwd(np.abs(g).astype(np.float64), ids1, ids2, num_nodes=n)
    big = torch.empty(need + 512, dtype=torch.uint8, device=dev)
    for ws in (None, big[:need // 2], big[1:need + 1]):
        gx = torch.zeros((n, D), device=dev)
        fsa.fsa_mean_bwd_ws(torch.from_numpy(g).to(dev), torch.from_numpy(ids1).to(dev), torch.from_numpy(ids2).to(dev),
                            grad_x=gx, workspace=ws)
        torch.cuda.synchronize()
        assert_close(to_f64(gx), ref, mag, 1e-5, "fallback")
