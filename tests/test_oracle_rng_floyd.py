"""Pins for the oracle's random-number generator and its without-replacement selection.

Philox is pinned to the known-answer vectors published with the generator; Floyd's selection is
pinned by exhaustive enumeration of its random choices (every k-subset must come out equally
often, which is the algorithm's textbook guarantee) and by a chi-square test with real Philox
words on rows of degree 7, 64 and 1000."""
import itertools
import math
import os
from collections import Counter

import numpy as np
import pytest

from conftest import GOLDEN
from oracle import reference as R


def _kat():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert R.philox4x32_10(ctr, key).tolist() == want


def _philox_bigint(ctr, key, rounds=10):
    """Philox4x32 from the SC'11 paper's definition with Python integers: per round two 32x32 -> 64
    bit products of counter words 0 and 2 with the multipliers M0, M1; the new counter is
    (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key is bumped by the Weyl constants."""
    M0, M1, W0, W1, mask = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85, 0xFFFFFFFF
    c0, c1, c2, c3 = [int(x) for x in ctr]
    k0, k1 = [int(x) for x in key]
    for _ in range(rounds):
        p0, p1 = M0 * c0, M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & mask, p1 & mask, ((p0 >> 32) ^ c3 ^ k1) & mask, p0 & mask
        k0, k1 = (k0 + W0) & mask, (k1 + W1) & mask
    return [c0, c1, c2, c3]


def test_philox_third_implementation_agrees():
    """A big-integer Python Philox written from the definition agrees with the oracle's C routine on
    the known-answer vectors and on 10^4 random (counter, key) pairs."""
    for ctr, key, want in _kat():
        assert _philox_bigint(ctr, key) == want
    rng = np.random.default_rng(11)
    for _ in range(10000):
        ctr = rng.integers(0, 1 << 32, 4, dtype=np.uint64).tolist()
        key = rng.integers(0, 1 << 32, 2, dtype=np.uint64).tolist()
        assert R.philox4x32_10(ctr, key).tolist() == _philox_bigint(ctr, key)


def test_philox_is_a_bijection_on_counters_and_keyed():
    key = [123, 456]
    outs = {tuple(R.philox4x32_10([c, 0, 0, 0], key).tolist()) for c in range(2000)}
    assert len(outs) == 2000
    assert R.philox4x32_10([1, 2, 3, 4], [5, 6]).tolist() != R.philox4x32_10([1, 2, 3, 4], [5, 7]).tolist()


def test_philox_word_keying():
    # counter = (v, iter lo, iter hi, layer * 65536 + draw // 4), key = (seed lo, seed hi)
    seed, it, layer, v = 0x1234567899ABCDEF, 0xA5A5A5A512345678, 2, 77777
    for draw in range(0, 23):
        blk = R.philox4x32_10([v, it & 0xFFFFFFFF, it >> 32, (layer << 16) | (draw // 4)],
                              [seed & 0xFFFFFFFF, seed >> 32])
        assert R.philox_word(seed, it, layer, v, draw) == int(blk[draw % 4])
    # every field matters
    base = R.philox_word(1, 2, 1, 3, 0)
    assert len({base, R.philox_word(2, 2, 1, 3, 0), R.philox_word(1, 3, 1, 3, 0),
                R.philox_word(1, 2, 0, 3, 0), R.philox_word(1, 2, 1, 4, 0),
                R.philox_word(1 << 32 | 1, 2, 1, 3, 0), R.philox_word(1, 1 << 32 | 2, 1, 3, 0)}) == 7


def _word_for(t, j):
    """A 32-bit word that the multiply-high rule maps to t in [0, j]."""
    w = -((-t * (1 << 32)) // (j + 1))  # ceil(t * 2^32 / (j+1))
    assert 0 <= w < (1 << 32) and (w * (j + 1)) >> 32 == t
    return w


@pytest.mark.parametrize("d,k", [(5, 3), (6, 2), (7, 4), (4, 3), (9, 1)])
def test_floyd_exhaustive_uniform_subsets(d, k):
    ranges = [range(d - k + i + 1) for i in range(k)]   # step i draws t in [0, j], j = d-k+i
    seen = Counter()
    for ts in itertools.product(*ranges):
        words = np.array([_word_for(t, d - k + i) for i, t in enumerate(ts)], np.uint32)
        chosen = R.floyd_select(d, k, words)
        assert len(set(chosen.tolist())) == k and chosen.min() >= 0 and chosen.max() < d
        # insertion order: step i inserts t unless t was inserted before, else j
        prev = set()
        for i, t in enumerate(ts):
            want = t if t not in prev else d - k + i
            assert chosen[i] == want
            prev.add(want)
        seen[frozenset(chosen.tolist())] += 1
    n_sub = math.comb(d, k)
    total = math.prod(len(r) for r in ranges)
    assert len(seen) == n_sub
    assert set(seen.values()) == {total // n_sub}


def test_multiply_high_range_mapping_is_even():
    # floor(w * m / 2^32) over all w hits each t in [0, m) either floor or ceil(2^32/m) times
    for m in (3, 7, 10, 1000):
        edges = [-((-t * (1 << 32)) // m) for t in range(m + 1)]
        sizes = {edges[t + 1] - edges[t] for t in range(m)}
        assert sizes <= {(1 << 32) // m, (1 << 32) // m + 1}


@pytest.mark.parametrize("d,k", [(7, 5), (64, 5), (64, 20), (1000, 20)])
def test_floyd_with_philox_is_uniform(d, k):
    """Each position is included with probability k/d, each pair with k(k-1)/(d(d-1))."""
    n_draws = 40000 if d <= 64 else 20000
    incl = np.zeros(d, np.int64)
    pair = np.zeros((d, d), np.int64) if d <= 64 else None
    v = 4242
    for it in range(n_draws):
        words = np.array([R.philox_word(99, it, 1, v, q) for q in range(k)], np.uint32)
        ch = R.floyd_select(d, k, words)
        incl[ch] += 1
        if pair is not None:
            pair[np.ix_(ch, ch)] += 1
    exp = n_draws * k / d
    chi2 = ((incl - exp) ** 2 / exp).sum()
    # inclusion counts are negatively correlated, which only lowers the statistic; use a loose
    # upper bound: mean d-1, sd sqrt(2(d-1)); allow 6 sigma
    assert chi2 < (d - 1) + 6 * math.sqrt(2 * (d - 1)), chi2
    if pair is not None:
        off = pair[~np.eye(d, dtype=bool)]
        pexp = n_draws * k * (k - 1) / (d * (d - 1))
        z = (off - pexp) / math.sqrt(pexp)
        assert np.abs(z).max() < 6.0
