"""Invariants of the oracle's fused forward on random CSR graphs (no GPU)."""
import numpy as np
from hypothesis import given, settings, strategies as st


def _graph(rng, n, max_deg):
    deg = rng.integers(0, max_deg + 1, size=n)
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    indices = rng.integers(0, n, size=int(indptr[-1])).astype(np.int32)
    return indptr, indices, deg


@settings(max_examples=60, deadline=None)
@given(st.integers(0, 2**32 - 1), st.integers(2, 40), st.integers(0, 30), st.integers(1, 12),
       st.integers(1, 12), st.integers(0, 2**64 - 1))
def test_forward_invariants(orc, gseed, n, max_deg, k1, k2, seed):
    rng = np.random.default_rng(gseed)
    indptr, indices, deg = _graph(rng, n, max_deg)
    D = 5
    x = rng.standard_normal((n, D))
    B = min(n, 9)
    seeds = rng.integers(0, n, size=B).astype(np.int32)   # duplicates allowed
    out1, _, ids1, _ = orc.sample_mean_fwd(indptr, indices, x, seeds, [k1], seed)
    out2, h1, ids1b, ids2 = orc.sample_mean_fwd(indptr, indices, x, seeds, [k1, k2], seed)
    # hop-0 draws do not depend on the number of hops
    assert (ids1 == ids1b).all()
    for b in range(B):
        r = int(seeds[b])
        row = indices[indptr[r]:indptr[r + 1]]
        cnt = min(k1, int(deg[r]))
        got = ids1[b]
        assert (got[cnt:] == -1).all() and (got[:cnt] >= 0).all()
        pos, ids, c = orc.sample_row(indptr, indices, r, 0, k1, seed)
        assert c == cnt and (ids == got).all()
        assert len(set(pos[:cnt].tolist())) == cnt and all(0 <= p < deg[r] for p in pos[:cnt])
        if deg[r] <= k1:
            assert got[:cnt].tolist() == row.tolist()
        # Prop. 1: the mean over exactly those rows
        want = x[got[:cnt]].mean(axis=0) if cnt else np.zeros(D)
        assert np.allclose(out1[b], want, rtol=1e-13, atol=1e-15)
        # 2-hop structure
        live = []
        for j in range(k1):
            if got[j] < 0:
                assert (ids2[b, j] == -1).all() and (h1[b, j] == 0).all()
                continue
            u = int(got[j])
            c2 = min(k2, int(deg[u]))
            w = ids2[b, j]
            assert (w[c2:] == -1).all() and (w[:c2] >= 0).all()
            _, wids, _ = orc.sample_row(indptr, indices, u, 1, k2, seed)
            assert (wids == w).all()
            if c2:
                assert np.allclose(h1[b, j], x[w[:c2]].mean(axis=0), rtol=1e-13, atol=1e-15)
                live.append(h1[b, j])
            else:
                assert (h1[b, j] == 0).all()
        want2 = np.mean(live, axis=0) if live else np.zeros(D)
        assert np.allclose(out2[b], want2, rtol=1e-13, atol=1e-15)
    # duplicate seeds give duplicate rows; outputs do not depend on batch order or size
    perm = rng.permutation(B)
    o_p, h_p, i1_p, i2_p = orc.sample_mean_fwd(indptr, indices, x, seeds[perm], [k1, k2], seed)
    assert (i1_p == ids1[perm]).all() and (i2_p == ids2[perm]).all()
    assert (o_p == out2[perm]).all() and (h_p == h1[perm]).all()


def test_same_inputs_same_ids_other_seed_other_ids(orc):
    rng = np.random.default_rng(1)
    indptr, indices, _ = _graph(rng, 300, 80)
    x = rng.standard_normal((300, 3))
    seeds = np.arange(300, dtype=np.int32)
    a = orc.sample_mean_fwd(indptr, indices, x, seeds, [5, 4], 77)
    b = orc.sample_mean_fwd(indptr, indices, x, seeds, [5, 4], 77)
    c = orc.sample_mean_fwd(indptr, indices, x, seeds, [5, 4], 78)
    assert (a[2] == b[2]).all() and (a[3] == b[3]).all() and (a[0] == b[0]).all()
    assert (a[2] != c[2]).any() and (a[3] != c[3]).any()


def test_int64_indptr_and_feature_types_agree(orc):
    rng = np.random.default_rng(2)
    indptr, indices, _ = _graph(rng, 200, 40)
    x32 = rng.standard_normal((200, 8)).astype(np.float32)
    seeds = rng.integers(0, 200, 50).astype(np.int32)
    a = orc.sample_mean_fwd(indptr, indices, x32, seeds, [6, 3], 5)
    b = orc.sample_mean_fwd(indptr.astype(np.int64), indices, x32.astype(np.float64), seeds, [6, 3], 5)
    for u, v in zip(a, b):
        assert (u == v).all()
    # bfloat16 storage: the oracle widens the bit patterns exactly
    bits = orc.round_to_bf16(x32.astype(np.float64))
    xb = orc.bf16_bits_to_f64(bits)
    c = orc.sample_mean_fwd(indptr, indices, bits, seeds, [6, 3], 5, bf16=True)
    d = orc.sample_mean_fwd(indptr, indices, xb, seeds, [6, 3], 5)
    assert (c[0] == d[0]).all() and (c[1] == d[1]).all() and (c[2] == d[2]).all()


def test_bf16_rounding_is_nearest_even(orc):
    import torch
    rng = np.random.default_rng(4)
    v = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38, 1e-40]])
    got = orc.round_to_bf16(v)
    # values exactly representable in float32 round the same way through torch's float->bf16
    v32 = v.astype(np.float32).astype(np.float64)
    want = torch.from_numpy(v32.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (orc.round_to_bf16(v32) == want).all()
    # and the direct rounding is the nearest representable value of the double itself
    back = orc.bf16_bits_to_f64(got)
    fin = np.isfinite(back) & (v != 0)
    half_ulp = 2.0 ** (np.maximum(np.floor(np.log2(np.abs(v[fin]))), -126) - 8)
    assert np.all(np.abs(back[fin] - v[fin]) <= half_ulp)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to the even significand (1.0)
    assert orc.round_to_bf16(np.array([1.00390625]))[0] == 0x3F80
    assert orc.round_to_bf16(np.array([1.01171875]))[0] == 0x3F82   # 1+3*2^-8 -> 1+2^-6
