"""Pins for the oracle's backward pass (no GPU): finite differences, the adjoint identity
and the transposed weight matrix built with scipy."""
import numpy as np
import scipy.sparse as sp


def _setup(orc, hops, seed=0):
    rng = np.random.default_rng(seed)
    n, D = 120, 4
    deg = rng.integers(0, 25, size=n)
    deg[rng.random(n) < 0.15] = 0
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    indices = rng.integers(0, n, size=int(indptr[-1])).astype(np.int32)
    x = rng.standard_normal((n, D))
    seeds = rng.integers(0, n, 40).astype(np.int32)
    fan = [6] if hops == 1 else [5, 4]
    out, h1, ids1, ids2 = orc.sample_mean_fwd(indptr, indices, x, seeds, fan, 17)
    return rng, n, D, x, ids1, ids2, out, h1


def test_backward_one_hop_finite_differences(orc):
    rng, n, D, x, ids1, _, out, _ = _setup(orc, 1)
    g = rng.standard_normal(out.shape)
    gx = orc.mean_bwd(g, ids1, num_nodes=n)
    loss = lambda xx: float((orc.mean_replay_fwd(xx, ids1)[0] * g).sum())
    eps = 1e-3
    for _ in range(60):
        r, d = int(rng.integers(n)), int(rng.integers(D))
        xp, xm = x.copy(), x.copy()
        xp[r, d] += eps
        xm[r, d] -= eps
        fd = (loss(xp) - loss(xm)) / (2 * eps)
        assert abs(fd - gx[r, d]) <= 1e-9 * max(1.0, abs(fd))


def test_backward_two_hop_finite_differences_with_h1_gradient(orc):
    rng, n, D, x, ids1, ids2, out, h1 = _setup(orc, 2)
    g = rng.standard_normal(out.shape)
    gh = rng.standard_normal(h1.shape)
    gx = orc.mean_bwd(g, ids1, ids2, gh, num_nodes=n)

    def loss(xx):
        o, h = orc.mean_replay_fwd(xx, ids1, ids2)
        return float((o * g).sum() + (h * gh).sum())
    eps = 1e-3
    touched = np.unique(ids2[ids2 >= 0])
    rows = list(rng.choice(touched, 40)) + list(rng.integers(0, n, 20))
    for r in rows:
        d = int(rng.integers(D))
        xp, xm = x.copy(), x.copy()
        xp[r, d] += eps
        xm[r, d] -= eps
        fd = (loss(xp) - loss(xm)) / (2 * eps)
        assert abs(fd - gx[r, d]) <= 1e-9 * max(1.0, abs(fd))
    # hop-1 nodes themselves receive nothing unless they are also somebody's leaf
    only_hop1 = np.setdiff1d(np.unique(ids1[ids1 >= 0]), touched)
    assert (gx[only_hop1] == 0).all()


def test_adjoint_identity(orc):
    for hops in (1, 2):
        rng, n, D, x, ids1, ids2, out, h1 = _setup(orc, hops, seed=hops)
        g = rng.standard_normal(out.shape)
        gh = rng.standard_normal(h1.shape) if hops == 2 else None
        gx = orc.mean_bwd(g, ids1, ids2, gh, num_nodes=n)
        lhs = (out * g).sum() + ((h1 * gh).sum() if hops == 2 else 0.0)
        assert abs(lhs - (x * gx).sum()) <= 1e-10 * max(1.0, abs(lhs))


def test_backward_is_transposed_weight_matrix(orc):
    rng, n, D, x, ids1, _, out, _ = _setup(orc, 1, seed=5)
    B, k = ids1.shape
    cnt = (ids1 >= 0).sum(axis=1)
    rows, cols, vals = [], [], []
    for b in range(B):
        for i in range(k):
            if ids1[b, i] >= 0:
                rows.append(b); cols.append(int(ids1[b, i])); vals.append(1.0 / cnt[b])
    S = sp.csr_matrix((vals, (rows, cols)), shape=(B, n))      # duplicates are summed
    assert np.allclose(S @ x, out, rtol=1e-12, atol=1e-14)
    g = rng.standard_normal(out.shape)
    assert np.allclose(orc.mean_bwd(g, ids1, num_nodes=n), S.T @ g, rtol=1e-12, atol=1e-14)


def test_backward_accumulates_into_grad_x(orc):
    rng, n, D, x, ids1, ids2, out, h1 = _setup(orc, 2, seed=6)
    g = rng.standard_normal(out.shape)
    once = orc.mean_bwd(g, ids1, ids2, num_nodes=n)
    twice = orc.mean_bwd(g, ids1, ids2, num_nodes=n, grad_x=once.copy())
    assert np.allclose(twice, 2 * once, rtol=1e-13, atol=0)
