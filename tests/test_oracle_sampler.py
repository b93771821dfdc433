"""Pins for the oracle's generator sampler (Alg. 1, Compress, sampling step: k distinct rows, uniform).

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


# ---- the bounded draw and its rejection branch.  The sampler itself only ever asks for ranges below 2^31, where a
# rejection has probability below 2^-33, so these pins ask for ranges of the order of 2^63, where a quarter to a half
# of the generator's outputs must be thrown away.

def _published_outputs():
    return [int(line) for line in open(GOLDEN) if line.strip() and not line.startswith("#")]


@pytest.mark.parametrize("u", [3 << 62, (1 << 63) + 12345, (1 << 63) - 1, (1 << 62) + 1, 5, 1])
def test_bounded_draw_on_the_published_stream(oracle, u):
    """Expected values come from the published splitmix64 outputs and exact integer arithmetic alone: outputs below
    2^64 mod u are skipped (each skip consumes one output), the others are reduced mod u."""
    pub = _published_outputs()
    cut = (1 << 64) % u
    want = [x % u for x in pub if x >= cut]
    if cut > 1 << 61:
        assert len(want) < len(pub)                   # the published stream really contains rejected outputs for this range
    got = oracle.bounded(1234567, u, len(want)).tolist()
    assert got == want


def test_bounded_draw_is_uniform_where_a_plain_remainder_is_not(oracle):
    """Range u = 3 * 2^62: without the rejection the lowest third [0, 2^62) would come up half of the time
    (2^64 = u + 2^62); with it every third comes up a third of the time."""
    u, trials = 3 << 62, 60_000
    draws = oracle.bounded(99, u, trials).astype(object)
    assert all(0 <= int(v) < u for v in draws[:1000])
    thirds = Counter(int(v) // (1 << 62) for v in draws)
    for t in range(3):
        assert abs(thirds[t] / trials - 1 / 3) < 6 * math.sqrt((1 / 3) * (2 / 3) / trials)


def test_bounded_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.bounded(0, 0, 4)


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
