"""Pins for the oracle's random-number layer (no GPU).

Philox4x32-10 is pinned by the published known-answer vectors; the bounded draw by its
counter/key layout, its range and its uniformity."""
import os

import numpy as np
import pytest
from scipy import stats

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            w = [int(t, 16) for t in line.split()]
            assert len(w) == 10
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(orc):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(orc.philox4x32_10(ctr, key)) == want


def test_philox_each_input_word_matters(orc):
    # flipping one bit of any counter or key word changes about half of the 128 output bits
    base_c, base_k = [1, 2, 3, 4], [5, 6]
    base = orc.philox4x32_10(base_c, base_k)
    for word in range(6):
        c, k = list(base_c), list(base_k)
        if word < 4:
            c[word] ^= 1 << 7
        else:
            k[word - 4] ^= 1 << 7
        got = orc.philox4x32_10(c, k)
        flipped = sum(bin(a ^ b).count("1") for a, b in zip(base, got))
        assert 32 <= flipped <= 96, (word, flipped)


def test_draw_layout_is_counter_node_hop_step_key_seed(orc):
    # draw = (word 0 of Philox(ctr=(node, hop, step, 0), key=(seed lo, seed hi)) * n) >> 32
    seed = 0x0123456789ABCDEF
    for node, hop, step, n in [(0, 0, 0, 1), (17, 1, 3, 10), (2**31 - 1, 1, 63, 2**31 - 1),
                               (123456, 0, 9, 4_000_000)]:
        r0 = orc.philox4x32_10([node, hop, step, 0], [seed & 0xFFFFFFFF, seed >> 32])[0]
        assert orc.draw(seed, node, hop, step, n) == (r0 * n) >> 32
    # the three counter fields are not interchangeable
    a = orc.draw(seed, 1, 0, 2, 2**31)
    assert a != orc.draw(seed, 2, 0, 1, 2**31)
    assert a != orc.draw(seed, 1, 2, 0, 2**31)
    assert a != orc.draw(seed ^ (1 << 40), 1, 0, 2, 2**31)


def test_draw_stays_in_range(orc):
    rng = np.random.default_rng(0)
    for n in [1, 2, 3, 7, 200, 21_700, 3_900_000, 2**31 - 1, 2**32 - 1]:
        for _ in range(200):
            node, step = int(rng.integers(0, 2**31)), int(rng.integers(0, 64))
            assert 0 <= orc.draw(5, node, 1, step, n) < n


def test_multiply_high_bias_bound():
    # exhaustive 16-bit analogue of the 32-bit map r -> (r*n) >> 32: every value of [0,n)
    # is hit floor(2^16/n) or ceil(2^16/n) times, i.e. relative bias <= n / 2^16.
    r = np.arange(1 << 16, dtype=np.uint64)
    for n in [1, 2, 3, 10, 255, 256, 257, 1000, 40000]:
        counts = np.bincount(((r * n) >> 16).astype(np.int64), minlength=n)
        assert counts.size == n
        assert set(np.unique(counts)) <= {(1 << 16) // n, -(-(1 << 16) // n)}


@pytest.mark.parametrize("n", [2, 5, 13])
def test_draw_is_uniform(orc, n):
    counts = np.zeros(n, dtype=np.int64)
    for node in range(6000):
        counts[orc.draw(42, node, 0, node % 7, n)] += 1
    assert stats.chisquare(counts).pvalue > 1e-4
