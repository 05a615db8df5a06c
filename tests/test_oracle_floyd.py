"""Pins for the oracle's sampler (no GPU): Floyd's selection is exactly uniform over
k-subsets (brute force over every draw tuple), and end to end (Philox -> draw -> Floyd ->
CSR row) it gives uniform subsets and the inclusion probability k/deg of Lemma 1."""
import itertools
import math

import numpy as np
import pytest
from scipy import stats


@pytest.mark.parametrize("deg,k", [(5, 2), (6, 3), (7, 4), (4, 3), (6, 1), (5, 4)])
def test_floyd_every_subset_exactly_k_factorial_times(orc, deg, k):
    ranges = [range(deg - k + i + 1) for i in range(k)]
    seen = {}
    total = 0
    for t in itertools.product(*ranges):
        pos = orc.floyd_select(deg, k, t)
        assert len(pos) == k
        assert len(set(pos.tolist())) == k
        assert all(0 <= p < deg for p in pos)
        key = frozenset(pos.tolist())
        seen[key] = seen.get(key, 0) + 1
        total += 1
    assert total == math.factorial(deg) // math.factorial(deg - k)
    assert len(seen) == math.comb(deg, k)
    assert set(seen.values()) == {math.factorial(k)}


def test_floyd_slot_order_and_collision_rule(orc):
    # step i draws from [0, deg-k+i]; a repeated draw is replaced by deg-k+i itself
    assert orc.floyd_select(10, 3, [4, 4, 4]).tolist() == [4, 8, 9]
    assert orc.floyd_select(10, 3, [7, 7, 8]).tolist() == [7, 8, 9]
    assert orc.floyd_select(10, 3, [0, 8, 9]).tolist() == [0, 8, 9]
    assert orc.floyd_select(10, 3, [2, 5, 1]).tolist() == [2, 5, 1]
    # a draw equal to an earlier replacement value also collides
    assert orc.floyd_select(10, 4, [3, 3, 7, 1]).tolist() == [3, 7, 8, 1]


def test_floyd_short_rows_take_everything(orc):
    assert orc.floyd_select(0, 5, [0] * 5).tolist() == []
    assert orc.floyd_select(3, 5, [9] * 5).tolist() == [0, 1, 2]
    assert orc.floyd_select(5, 5, [9] * 5).tolist() == [0, 1, 2, 3, 4]


def _single_row(deg):
    indptr = np.array([0, deg], dtype=np.int32)
    indices = np.arange(100, 100 + deg, dtype=np.int32)
    return indptr, indices


@pytest.mark.parametrize("deg,k", [(5, 2), (6, 3), (8, 4)])
def test_end_to_end_subsets_uniform_over_seeds(orc, deg, k):
    indptr, indices = _single_row(deg)
    subsets = {s: i for i, s in enumerate(itertools.combinations(range(deg), k))}
    counts = np.zeros(len(subsets), dtype=np.int64)
    incl = np.zeros(deg, dtype=np.int64)
    M = 40_000
    for seed in range(M):
        pos, ids, cnt = orc.sample_row(indptr, indices, 0, 0, k, seed * 0x9E3779B1 + 11)
        assert cnt == k
        assert (ids[:k] == indices[pos[:k]]).all()
        counts[subsets[tuple(sorted(pos[:k].tolist()))]] += 1
        incl[pos[:k]] += 1
    assert stats.chisquare(counts).pvalue > 1e-4
    # Lemma 1: each neighbor is included with probability k / deg
    p = k / deg
    sigma = math.sqrt(p * (1 - p) / M)
    assert np.all(np.abs(incl / M - p) < 5 * sigma)


def test_inclusion_probability_over_nodes_and_hops(orc):
    # vary node id and hop instead of the seed: the counter fields give independent streams
    deg, k = 9, 4
    M = 20_000
    indptr = np.arange(0, (M + 1) * deg, deg, dtype=np.int64)
    indices = np.tile(np.arange(deg, dtype=np.int32), M)
    for hop in (0, 1):
        incl = np.zeros(deg, dtype=np.int64)
        for node in range(M):
            pos, _, _ = orc.sample_row(indptr, indices, node, hop, k, 7)
            incl[pos[:k]] += 1
        p = k / deg
        assert np.all(np.abs(incl / M - p) < 5 * math.sqrt(p * (1 - p) / M))


def test_sample_row_is_floyd_on_the_documented_draws(orc):
    # J = deg-k+i, t_i = draw(seed, node, hop, i, J+1), positions = floyd(deg, k, t)
    rng = np.random.default_rng(3)
    deg_list = rng.integers(0, 60, size=50)
    indptr = np.concatenate([[0], np.cumsum(deg_list)]).astype(np.int32)
    indices = rng.integers(0, 50, size=int(indptr[-1])).astype(np.int32)
    for node in range(50):
        for hop, k, seed in [(0, 7, 99), (1, 25, 2**63 + 5)]:
            deg = int(deg_list[node])
            pos, ids, cnt = orc.sample_row(indptr, indices, node, hop, k, seed)
            assert cnt == min(k, deg)
            if deg <= k:
                want = list(range(deg))
            else:
                t = [orc.draw(seed, node, hop, i, deg - k + i + 1) for i in range(k)]
                want = orc.floyd_select(deg, k, t).tolist()
            assert pos[:cnt].tolist() == want
            assert (pos[cnt:] == -1).all() and (ids[cnt:] == -1).all()
            assert ids[:cnt].tolist() == [int(indices[indptr[node] + p]) for p in want]
