"""Pins for the oracle's generator sampler (Alg. 1, Compress: "sample indices uniformly without replacement").

The paper fixes only the distribution, so the pins are: the published splitmix64
vectors, the permutation property at k = b, and the uniform-without-replacement
law that the proof of Lemma 2 relies on (Pr[all k draws miss a set of size s] =
C(b-s,k)/C(b,k)).  The index stream itself is fixed by this build's own
specification: "parity unpinned" by the paper.
"""
import math
import os
from collections import Counter

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed1234567.txt")


def test_splitmix64_published_vectors(oracle):
    want = [int(line) for line in open(GOLDEN) if line.strip() and not line.startswith("#")]
    got = [int(v) for v in oracle.splitmix64(1234567, len(want))]
    assert got == want


@pytest.mark.parametrize("b", [1, 2, 7, 64, 2048])
def test_full_draw_is_a_permutation(oracle, b):
    idx = oracle.sample(b, b, seed=b + 11)
    assert sorted(idx.tolist()) == list(range(b))


@pytest.mark.parametrize("b,k", [(8, 3), (100, 17), (65536, 128), (16384, 1024)])
def test_distinct_in_range_deterministic_prefix(oracle, b, k):
    a = oracle.sample(b, k, seed=5)
    assert a.dtype == np.int32 and a.shape == (k,)
    assert len(set(a.tolist())) == k and a.min() >= 0 and a.max() < b
    assert np.array_equal(a, oracle.sample(b, k, seed=5))
    assert not np.array_equal(a, oracle.sample(b, k, seed=6))
    # draw t only depends on the draws before it, so a longer draw extends a shorter one
    longer = oracle.sample(b, min(b, k + 5), seed=5)
    assert np.array_equal(longer[:k], a)


def test_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.sample(4, 5, 0)
    with pytest.raises(ValueError):
        oracle.sample(4, 0, 0)


def test_every_ordered_draw_equally_likely(oracle):
    """b = 8, k = 3: 336 ordered outcomes; chi-square against the uniform law."""
    b, k, trials = 8, 3, 100_000
    counts = Counter(tuple(oracle.sample(b, k, seed).tolist()) for seed in range(trials))
    outcomes = b * (b - 1) * (b - 2)
    assert len(counts) == outcomes
    expect = trials / outcomes
    chi2 = sum((c - expect) ** 2 / expect for c in counts.values())
    # dof = 335: mean 335, sd ~ 25.9; 6 sd is a failure probability far below 1e-6
    assert chi2 < 335 + 6 * math.sqrt(2 * 335)
    # inclusion frequency of every index is k/b
    incl = Counter()
    for tup, c in counts.items():
        for v in tup:
            incl[v] += c
    for v in range(b):
        assert abs(incl[v] / trials - k / b) < 6 * math.sqrt((k / b) * (1 - k / b) / trials)


def test_miss_probability_matches_hypergeometric(oracle):
    """Proof of Lemma 2: the chance that all k generators fall outside a set of size s is C(b-s,k)/C(b,k)."""
    b, k, s, trials = 20, 5, 6, 60_000
    target = set(range(3, 3 + s))
    miss = sum(1 for seed in range(trials) if target.isdisjoint(oracle.sample(b, k, 1_000_003 * seed + 17).tolist()))
    p = math.comb(b - s, k) / math.comb(b, k)
    assert abs(miss / trials - p) < 6 * math.sqrt(p * (1 - p) / trials)


def _python_restatement(b, k, seed):
    """The specification written out again with Python integers (sparse map instead of a full array)."""
    M = (1 << 64) - 1
    state = seed & M
    moved = {}
    out = []
    for t in range(k):
        u = b - t
        reject_below = ((1 << 64) - u) % u          # 2^64 mod u
        while True:
            state = (state + 0x9E3779B97F4A7C15) & M
            z = state
            z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
            z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
            z ^= z >> 31
            if z >= reject_below:
                break
        r = t + z % u
        vt, vr = moved.get(t, t), moved.get(r, r)
        moved[t], moved[r] = vr, vt
        out.append(vr)
    return out


@pytest.mark.parametrize("b,k,seed", [(10, 10, 0), (8192, 16, 0), (65536, 128, 3), (16384, 1024, 2**63 + 5), (3, 2, 2**64 - 1)])
def test_matches_the_written_specification(oracle, b, k, seed):
    assert oracle.sample(b, k, seed).tolist() == _python_restatement(b, k, seed)
