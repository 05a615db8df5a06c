"""Pins for the oracle's weighted-mean extension (no GPU)."""
import numpy as np
import scipy.sparse as sp


def _graph(rng, n, max_deg, zero_frac=0.2):
    deg = rng.integers(0, max_deg + 1, size=n)
    deg[rng.random(n) < zero_frac] = 0
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    indices = rng.integers(0, n, size=int(indptr[-1])).astype(np.int32)
    return indptr, indices, deg


def _norm_rows(A):
    d = np.asarray(A.sum(axis=1)).ravel()
    inv = np.divide(1.0, d, out=np.zeros_like(d), where=d > 0)
    return sp.diags(inv) @ A


def test_unit_weights_reproduce_the_unweighted_functions_bit_for_bit(orc):
    rng = np.random.default_rng(0)
    n = 400
    indptr, indices, _ = _graph(rng, n, 40)
    x = rng.standard_normal((n, 6)).astype(np.float32)
    ones = np.ones(indices.size, dtype=np.float32)
    seeds = rng.integers(0, n, 150).astype(np.int32)
    for fan in ([7], [6, 4]):
        a = orc.sample_mean_fwd(indptr, indices, x, seeds, fan, 21)
        b = orc.sample_wmean_fwd(indptr, indices, ones, x, seeds, fan, 21)
        assert (a[0] == b[0]).all() and (a[2] == b[2]).all()
        if len(fan) == 2:
            assert (a[1] == b[1]).all() and (a[3] == b[3]).all()
        assert ((b[4] == 1) == (b[2] >= 0)).all() and (b[4][b[2] < 0] == 0).all()
        g = rng.standard_normal(a[0].shape)
        gh = rng.standard_normal(a[1].shape) if len(fan) == 2 else None
        ga = orc.mean_bwd(g, a[2], a[3], gh, num_nodes=n)
        gb = orc.wmean_bwd(g, b[2], b[4], b[3], b[5], gh, num_nodes=n)
        assert np.allclose(ga, gb, rtol=1e-12, atol=1e-15)    # same weights, different rounding order


def test_emitted_weights_are_the_sampled_edge_slots(orc):
    rng = np.random.default_rng(1)
    n = 300
    indptr, indices, deg = _graph(rng, n, 50, zero_frac=0.1)
    ew = rng.random(indices.size).astype(np.float32) + 0.1
    x = rng.standard_normal((n, 3))
    seeds = np.arange(n, dtype=np.int32)
    out, h1, ids1, ids2, w1, w2 = orc.sample_wmean_fwd(indptr, indices, ew, x, seeds, [8, 5], 3)
    for b in range(n):
        pos, ids, cnt = orc.sample_row(indptr, indices, b, 0, 8, 3)
        assert (ids == ids1[b]).all()
        assert np.array_equal(w1[b, :cnt], ew[indptr[b] + pos[:cnt]]) and (w1[b, cnt:] == 0).all()
        for j in range(cnt):
            u = int(ids1[b, j])
            p2, i2, c2 = orc.sample_row(indptr, indices, u, 1, 5, 3)
            assert (i2 == ids2[b, j]).all()
            assert np.array_equal(w2[b, j, :c2], ew[indptr[u] + p2[:c2]]) and (w2[b, j, c2:] == 0).all()


def test_full_fanout_reduces_to_weighted_adjacency_products(orc):
    rng = np.random.default_rng(2)
    n, D = 250, 5
    indptr, indices, deg = _graph(rng, n, 14, zero_frac=0.3)
    ew = (rng.random(indices.size) * (rng.random(indices.size) > 0.15)).astype(np.float32)   # some zero weights
    x = rng.standard_normal((n, D))
    Aw = sp.csr_matrix((ew.astype(np.float64), indices, indptr), shape=(n, n))     # duplicates summed
    PX = _norm_rows(Aw) @ x
    seeds = np.arange(n, dtype=np.int32)
    out1 = orc.sample_wmean_fwd(indptr, indices, ew, x, seeds, [14], 5)[0]
    assert np.allclose(out1, PX, rtol=1e-12, atol=1e-14)
    # 2-hop: hop-1 nodes whose weighted row sum is zero leave the outer sum and divisor
    rowsum = np.asarray(Aw.sum(axis=1)).ravel()
    takes_part = sp.diags((rowsum > 0).astype(np.float64))
    want = _norm_rows(Aw @ takes_part) @ PX
    out2, h1, ids1, ids2, w1, w2 = orc.sample_wmean_fwd(indptr, indices, ew, x, seeds, [14, 14], 5)
    assert np.allclose(out2, want, rtol=1e-12, atol=1e-14)
    for b in range(0, n, 7):
        for j in range(14):
            u = ids1[b, j]
            assert np.allclose(h1[b, j], PX[u] if u >= 0 else 0.0, rtol=1e-12, atol=1e-14)


def test_scale_invariance_and_zero_weights(orc):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((30, 4))
    ids1 = np.array([[3, 5, 9, -1]], dtype=np.int32)
    w1 = np.array([[2.0, 0.0, 6.0, 123.0]], dtype=np.float32)     # the padded slot's weight is ignored
    out, _ = orc.wmean_replay_fwd(x, ids1, w1)
    assert np.allclose(out[0], (2 * x[3] + 6 * x[9]) / 8)
    out_scaled, _ = orc.wmean_replay_fwd(x, ids1, w1 * 7)
    assert np.allclose(out, out_scaled, rtol=1e-14)
    assert (orc.wmean_replay_fwd(x, ids1, np.zeros_like(w1))[0] == 0).all()
    ids2 = np.array([[[1, 2], [3, -1], [4, 5], [6, 7]]], dtype=np.int32)
    w2 = np.array([[[1.0, 3.0], [0.0, 9.0], [2.0, 2.0], [1.0, 1.0]]], dtype=np.float32)
    out, h1 = orc.wmean_replay_fwd(x, ids1, w1, ids2, w2)
    assert np.allclose(h1[0, 0], (x[1] + 3 * x[2]) / 4)
    assert (h1[0, 1] == 0).all()                                   # its only valid leaf has weight 0
    assert np.allclose(h1[0, 2], (x[4] + x[5]) / 2) and (h1[0, 3] == 0).all()
    assert np.allclose(out[0], (2 * h1[0, 0] + 6 * h1[0, 2]) / 8)  # slot 1 (empty) and slot 3 (padded) left out


def test_weighted_backward_finite_differences_and_adjoint(orc):
    rng = np.random.default_rng(4)
    n, D = 90, 3
    indptr, indices, _ = _graph(rng, n, 20)
    ew = (rng.random(indices.size) * (rng.random(indices.size) > 0.1)).astype(np.float32)
    x = rng.standard_normal((n, D))
    seeds = rng.integers(0, n, 30).astype(np.int32)
    for fan in ([5], [4, 3]):
        out, h1, ids1, ids2, w1, w2 = orc.sample_wmean_fwd(indptr, indices, ew, x, seeds, fan, 8)
        g = rng.standard_normal(out.shape)
        gh = rng.standard_normal(h1.shape) if len(fan) == 2 else None
        gx = orc.wmean_bwd(g, ids1, w1, ids2, w2, gh, num_nodes=n)

        def loss(xx):
            o, h = orc.wmean_replay_fwd(xx, ids1, w1, ids2, w2)
            return float((o * g).sum() + ((h * gh).sum() if gh is not None else 0.0))
        lhs = loss(x)
        assert abs(lhs - (x * gx).sum()) <= 1e-10 * max(1.0, abs(lhs))       # linear map: <f(x),g> = <x,f^T g>
        eps = 1e-3
        for _ in range(40):
            r, d = int(rng.integers(n)), int(rng.integers(D))
            xp, xm = x.copy(), x.copy()
            xp[r, d] += eps
            xm[r, d] -= eps
            fd = (loss(xp) - loss(xm)) / (2 * eps)
            assert abs(fd - gx[r, d]) <= 1e-9 * max(1.0, abs(fd))
