"""Pins of the oracle's three-hop functions (no GPU).

- A fanout at least as large as every degree keeps whole rows, so the nested mean reduces to
  products with the adjacency matrix that scipy computes independently, empty neighborhoods
  leaving the sum and the divisor level by level.
- Every hop's IDs are the single-row sampler's (pinned elsewhere) with hop counters 0, 1, 2.
- For general fanouts the forward equals materialise-then-mean written with numpy (Prop. 1).
- The forward is linear in X, so <G, f(X)> = <f^T(G), X> for every output (adjoint identity),
  and a finite difference in one coordinate of X moves the loss by the gradient's entry.
- With k1 = 1 and a single neighbor the outer level is the identity and the result is the
  two-hop function of that neighbor with shifted hop counters: checked through the IDs and
  against numpy, not by calling the two-hop oracle."""
import numpy as np
import scipy.sparse as sp


def _graph(rng, n, max_deg, zero_frac=0.25):
    deg = rng.integers(0, max_deg + 1, size=n)
    deg[rng.random(n) < zero_frac] = 0
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    indices = rng.integers(0, n, size=int(indptr[-1])).astype(np.int32)
    return indptr, indices, deg


def _masked_mean(A, live, y):
    """Row r: mean of y[v] over the neighbors v of r (with multiplicity) that are live."""
    num = A @ (y * live[:, None])
    den = A @ live
    out = np.divide(num, den[:, None], out=np.zeros_like(num), where=den[:, None] > 0)
    return out, den


def test_full_fanout_is_three_nested_adjacency_products(orc):
    rng = np.random.default_rng(0)
    n, D, K = 250, 5, 9
    indptr, indices, deg = _graph(rng, n, K)
    x = rng.standard_normal((n, D))
    A = sp.csr_matrix((np.ones(indices.size), indices, indptr), shape=(n, n))
    ones = np.ones(n)
    y3, d3 = _masked_mean(A, ones, x)                   # leaf means; d3 = degree
    y2, d2 = _masked_mean(A, (d3 > 0).astype(float), y3)
    y1, d1 = _masked_mean(A, (d2 > 0).astype(float), y2)
    m1, _ = _masked_mean(A, ones, x)
    seeds = np.arange(n, dtype=np.int32)
    r = orc.sample_mean3_fwd(indptr, indices, x, seeds, [K, K, K], 5)
    assert np.allclose(r["out"], y1, rtol=1e-12, atol=1e-14)
    assert np.allclose(r["out_m1"], m1, rtol=1e-12, atol=1e-14)
    for b in range(0, n, 7):
        for j in range(K):
            u = r["ids1"][b, j]
            assert np.allclose(r["out_h1"][b, j], y2[u] if u >= 0 else 0.0, rtol=1e-12, atol=1e-14)
            assert r["cnt2"][b, j] == (d2[u] if u >= 0 else 0)
            for i in range(K):
                v = r["ids2"][b, j, i]
                assert np.allclose(r["out_h2"][b, j, i], y3[v] if v >= 0 else 0.0, rtol=1e-12, atol=1e-14)
    # the skipping rule is exercised at both levels
    assert ((r["ids2"] >= 0).sum(2) > r["cnt2"]).any()
    assert ((r["ids1"] >= 0).sum(1) > (r["cnt2"] > 0).sum(1)).any()


def test_ids_come_from_the_row_sampler_with_hop_counters_0_1_2(orc):
    rng = np.random.default_rng(1)
    n = 300
    indptr, indices, deg = _graph(rng, n, 40)
    x = rng.standard_normal((n, 2))
    seeds = rng.permutation(n)[:40].astype(np.int32)
    k1, k2, k3 = 4, 3, 5
    r = orc.sample_mean3_fwd(indptr, indices, x, seeds, [k1, k2, k3], 2**40 + 3)
    for b, s in enumerate(seeds):
        _, U, _ = orc.sample_row(indptr, indices, int(s), 0, k1, 2**40 + 3)
        assert np.array_equal(r["ids1"][b], U)
        for j in range(k1):
            if U[j] < 0:
                assert (r["ids2"][b, j] == -1).all() and (r["ids3"][b, j] == -1).all()
                continue
            _, V, _ = orc.sample_row(indptr, indices, int(U[j]), 1, k2, 2**40 + 3)
            assert np.array_equal(r["ids2"][b, j], V)
            for i in range(k2):
                if V[i] < 0:
                    assert (r["ids3"][b, j, i] == -1).all()
                else:
                    _, W, _ = orc.sample_row(indptr, indices, int(V[i]), 2, k3, 2**40 + 3)
                    assert np.array_equal(r["ids3"][b, j, i], W)


def _numpy_three_hop(x, ids1, ids2, ids3):
    B, k1, k2, k3 = ids3.shape
    D = x.shape[1]
    out, h1, h2 = np.zeros((B, D)), np.zeros((B, k1, D)), np.zeros((B, k1, k2, D))
    for b in range(B):
        mids = []
        for j in range(k1):
            leaves = []
            for i in range(k2):
                w = ids3[b, j, i]
                w = w[w >= 0]
                if ids1[b, j] >= 0 and ids2[b, j, i] >= 0 and w.size:
                    h2[b, j, i] = x[w].mean(0)
                    leaves.append(h2[b, j, i])
            if leaves:
                h1[b, j] = np.mean(leaves, axis=0)
                mids.append(h1[b, j])
        if mids:
            out[b] = np.mean(mids, axis=0)
    return out, h1, h2


def test_forward_and_replay_equal_materialise_then_mean(orc):
    rng = np.random.default_rng(2)
    n, D = 200, 6
    indptr, indices, deg = _graph(rng, n, 25)
    x = rng.standard_normal((n, D))
    seeds = rng.permutation(n)[:60].astype(np.int32)
    r = orc.sample_mean3_fwd(indptr, indices, x, seeds, [5, 4, 3], 77)
    out, h1, h2 = _numpy_three_hop(x, r["ids1"], r["ids2"], r["ids3"])
    assert np.allclose(r["out"], out, rtol=1e-12, atol=1e-14)
    assert np.allclose(r["out_h1"], h1, rtol=1e-12, atol=1e-14)
    assert np.allclose(r["out_h2"], h2, rtol=1e-12, atol=1e-14)
    # replay with holes punched anywhere in the saved IDs
    ids1, ids2, ids3 = r["ids1"].copy(), r["ids2"].copy(), r["ids3"].copy()
    ids3[rng.random(ids3.shape) < 0.3] = -1
    ids2[rng.random(ids2.shape) < 0.2] = -1
    ids1[rng.random(ids1.shape) < 0.2] = -1
    rp = orc.mean3_replay_fwd(x, ids1, ids2, ids3)
    out, h1, h2 = _numpy_three_hop(x, ids1, ids2, ids3)
    assert np.allclose(rp["out"], out, rtol=1e-12, atol=1e-14)
    assert np.allclose(rp["out_h1"], h1, rtol=1e-12, atol=1e-14)
    assert np.allclose(rp["out_h2"], h2, rtol=1e-12, atol=1e-14)
    m = ids1 >= 0
    want_m1 = np.stack([x[ids1[b][m[b]]].mean(0) if m[b].any() else np.zeros(D) for b in range(len(seeds))])
    assert np.allclose(rp["out_m1"], want_m1, rtol=1e-12, atol=1e-14)


def test_backward_adjoint_identity_and_finite_differences(orc):
    rng = np.random.default_rng(3)
    n, D = 120, 3
    indptr, indices, deg = _graph(rng, n, 20)
    x = rng.standard_normal((n, D))
    seeds = rng.permutation(n)[:50].astype(np.int32)
    r = orc.sample_mean3_fwd(indptr, indices, x, seeds, [4, 3, 3], 1)
    ids = (r["ids1"], r["ids2"], r["ids3"])
    G = {k: rng.standard_normal(r[k].shape) for k in ("out", "out_h1", "out_h2", "out_m1")}
    for use in (("out",), ("out", "out_h1"), ("out", "out_h2"), ("out", "out_m1"), ("out", "out_h1", "out_h2", "out_m1")):
        gx = orc.mean3_bwd(G["out"] if "out" in use else np.zeros_like(G["out"]), *ids,
                           grad_h1=G["out_h1"] if "out_h1" in use else None,
                           grad_h2=G["out_h2"] if "out_h2" in use else None,
                           grad_m1=G["out_m1"] if "out_m1" in use else None, num_nodes=n)
        lhs = sum((G[k] * r[k]).sum() for k in use)
        assert np.isclose(lhs, (gx * x).sum(), rtol=1e-11), use
        # central difference in a few coordinates (the map is linear, so it is exact up to rounding)
        for _ in range(5):
            a, d = rng.integers(n), rng.integers(D)
            xp, xm = x.copy(), x.copy()
            xp[a, d] += 0.5
            xm[a, d] -= 0.5
            fp = orc.mean3_replay_fwd(xp, *ids)
            fm = orc.mean3_replay_fwd(xm, *ids)
            diff = sum((G[k] * (fp[k] - fm[k])).sum() for k in use)
            assert np.isclose(diff, gx[a, d], rtol=1e-9, atol=1e-12), use


def test_chain_graph_by_hand(orc):
    """0 -> {1} -> {2, 3} -> leaves; node 3 has no neighbors: by hand,
    out_h2[0,0,:] = (mean(x[4], x[5]), 0), cnt2 = 1, out = out_h1 = mean(x[4], x[5])."""
    indptr = np.array([0, 1, 3, 5, 5, 5, 5], dtype=np.int32)
    indices = np.array([1, 2, 3, 4, 5], dtype=np.int32)
    x = np.arange(12, dtype=np.float64).reshape(6, 2)
    r = orc.sample_mean3_fwd(indptr, indices, x, np.array([0], dtype=np.int32), [2, 2, 2], 0)
    want = (x[4] + x[5]) / 2
    assert np.array_equal(r["ids1"], [[1, -1]])
    assert np.array_equal(r["ids2"][0, 0], [2, 3]) and np.array_equal(r["ids3"][0, 0], [[4, 5], [-1, -1]])
    assert np.array_equal(r["cnt2"], [[1, 0]])
    assert np.allclose(r["out"][0], want) and np.allclose(r["out_h1"][0, 0], want)
    assert np.allclose(r["out_h2"][0, 0, 0], want) and (r["out_h2"][0, 0, 1] == 0).all()
    assert np.allclose(r["out_m1"][0], x[1])
    gx = orc.mean3_bwd(np.ones((1, 2)), r["ids1"], r["ids2"], r["ids3"], num_nodes=6)
    assert np.allclose(gx[4], 0.5) and np.allclose(gx[5], 0.5) and np.allclose(gx[:4], 0)
