"""Pins for the oracle's neighbourhood condition (Eq. 2) and normalisation factor beta (Sec. 3.2).

Every check is written with numpy from the paper's statement of the condition, from the textbook
column-row-sampling estimator that PAMM reduces to at eps = 0 (Sec. 4.1), or from the error bound of
Sec. 3.2.1; none re-uses the oracle's code.
"""
import itertools

import numpy as np
import pytest


def _rng(seed):
    return np.random.default_rng(seed)


def _clustered(b, n, centres, sigma, seed):
    g = _rng(seed)
    mu = g.standard_normal((centres, n))
    z = g.integers(0, centres, b)
    s = g.uniform(0.5, 2.0, b) * g.choice([-1.0, 1.0], b)
    return mu[z] * s[:, None] + sigma * g.standard_normal((b, n))


def test_infinite_tolerance_is_the_unconditioned_path(oracle):
    X = _clustered(300, 24, 10, 0.2, 0)
    base = oracle.compress(X, 7, seed=3)
    for eps in (float("inf"), 1e9, 1.0):         # eps >= 1 can drop nothing: the residual of a projection never exceeds the norm
        c = oracle.compress(X, 7, seed=3, eps=eps)
        assert c.eta == 0 and c.beta == 1.0
        assert np.array_equal(c.f, base.f) and np.array_equal(c.alpha, base.alpha)


@pytest.mark.parametrize("eps", [0.0, 0.05, 0.2, 0.5, 0.9])
def test_kept_rows_are_those_of_the_neighbourhood_condition(oracle, eps):
    """Eq. 2 written out: row i is kept iff ||A_i - alpha_i C_f(i)||_2 <= eps ||A_i||_2."""
    X = _clustered(400, 20, 12, 0.15, 1)
    free = oracle.compress(X, 9, seed=5)                     # unmasked coefficients
    c = oracle.compress(X, 9, seed=5, eps=eps)
    C = X[free.idx]
    e = np.linalg.norm(X - free.alpha[:, None] * C[free.f], axis=1)
    na = np.linalg.norm(X, axis=1)
    margin = e - eps * na
    clear = (np.abs(margin) > 1e-9 * na) | (e == 0.0)        # not on the boundary itself (a zero residual is unambiguous)
    kept = margin <= 0
    assert clear.all() and np.all(free.alpha != 0)           # continuous data: nobody on the boundary, no zero coefficient
    assert np.array_equal(c.alpha != 0, kept)
    assert np.array_equal(c.f, free.f)                       # a dropped row keeps its generator (Alg. 1 only zeroes alpha)
    assert np.array_equal(c.alpha[kept], free.alpha[kept])
    assert c.eta == int(np.sum(~kept))
    assert c.beta == pytest.approx(400 / (400 - c.eta))
    # the same condition through Lemma 1's identity: kept iff csim^2 >= 1 - eps^2
    csim2 = free.best / na ** 2
    assert np.array_equal((csim2 >= 1 - eps ** 2 - 1e-12)[clear], kept[clear])      # 1e-12: a generator's own csim^2 rounds around 1
    assert np.allclose(c.resid, e, rtol=1e-12, atol=1e-12) and np.allclose(c.rownorm, na, rtol=1e-14)


def test_kept_set_grows_with_the_tolerance(oracle):
    X = _clustered(500, 16, 20, 0.3, 2)
    prev = None
    for eps in (0.0, 0.1, 0.3, 0.5, 0.7, 0.95, 1.0):
        c = oracle.compress(X, 11, seed=1, eps=eps)
        kept = c.alpha != 0
        if prev is not None:
            assert np.all(kept[prev])                         # monotone
        prev = kept
    assert prev.all()


def test_zero_tolerance_is_uniform_column_row_sampling(oracle):
    """eps = 0 keeps exactly the sampled rows (generic rows: nobody else lies on a generator's line), with
    alpha = 1, beta = b / k, so Otilde = (b/k) sum_{i in I} A_i^T B_i (Sec. 4.1, Uniform-CRS)."""
    g = _rng(3)
    b, n, m, k = 60, 9, 7, 8
    A = g.standard_normal((b, n))
    B = g.standard_normal((b, m))
    c = oracle.compress(A, k, seed=11, eps=0.0)
    kept = np.nonzero(c.alpha)[0]
    assert sorted(kept.tolist()) == sorted(c.idx.tolist())
    assert np.all(c.alpha[kept] == 1.0)
    assert c.eta == b - k and c.beta == pytest.approx(b / k)
    _, O = oracle.grad(c.C, c.f, c.alpha, B, beta=c.beta)
    crs = (b / k) * sum(np.outer(A[i], B[i]) for i in c.idx)
    assert np.allclose(O, crs, rtol=1e-12, atol=1e-12)


def test_beta_makes_column_row_sampling_unbiased(oracle):
    """Sec. 3.2: beta is chosen so that E[Otilde] = O.  At eps = 0 this is exact: the mean of Otilde over ALL
    k-subsets of the rows (each equally likely under uniform sampling without replacement) is A^T B."""
    g = _rng(4)
    b, n, m, k = 7, 4, 3, 3
    A = g.standard_normal((b, n))
    B = g.standard_normal((b, m))
    acc = np.zeros((n, m))
    count = 0
    for I in itertools.combinations(range(b), k):
        c = oracle.compress(A, k, idx=np.array(I, dtype=np.int32), eps=0.0)
        _, O = oracle.grad(c.C, c.f, c.alpha, B, beta=c.beta)
        acc += O
        count += 1
    assert count == 35
    assert np.allclose(acc / count, A.T @ B, rtol=1e-12, atol=1e-12)
    # without beta the same mean underestimates by exactly k/b
    c = oracle.compress(A, k, idx=np.array([0, 1, 2], dtype=np.int32), eps=0.0)
    _, O1 = oracle.grad(c.C, c.f, c.alpha, B)
    _, Ob = oracle.grad(c.C, c.f, c.alpha, B, beta=c.beta)
    assert np.allclose(Ob, (b / k) * O1, rtol=1e-14)


@pytest.mark.parametrize("eps", [0.0, 0.2, 0.6])
def test_error_bound_with_dropped_rows(oracle, eps):
    """Sec. 3.2.1 (the un-normalised estimate, beta = 1):
    ||O - A~^T B||_F^2 <= ||B||_2^2 (eps^2 ||A_I||_F^2 + ||A_Ibar||_F^2),  and  ||A - A~||_F^2 <= eps^2 ||A_I||_F^2 + ||A_Ibar||_F^2."""
    X = _clustered(240, 14, 8, 0.25, 5)
    g = _rng(6)
    B = g.standard_normal((240, 10))
    c = oracle.compress(X, 6, seed=2, eps=eps)
    kept = c.alpha != 0
    At = c.alpha[:, None] * c.C[c.f]
    rhs_a = eps ** 2 * np.sum(X[kept] ** 2) + np.sum(X[~kept] ** 2)
    assert np.sum((X - At) ** 2) <= rhs_a * (1 + 1e-12) + 1e-12
    _, O1 = oracle.grad(c.C, c.f, c.alpha, B)
    lhs = np.sum((X.T @ B - O1) ** 2)
    assert lhs <= np.linalg.norm(B, 2) ** 2 * rhs_a * (1 + 1e-12) + 1e-12
    assert np.allclose(O1, At.T @ B, rtol=1e-11, atol=1e-11)             # regrouping holds with dropped rows too


def test_collinear_rows_survive_zero_tolerance(oracle):
    """Exact multiples (power-of-two scales, either sign) and exact copies of a generator have zero residual."""
    g = _rng(7)
    A = g.standard_normal((12, 6)).astype(np.float32)
    A[4] = 2.0 * A[1]
    A[5] = -0.5 * A[1]
    A[6] = A[2]
    A[7] = 0.0
    c = oracle.compress(A, 2, idx=np.array([1, 2], dtype=np.int32), eps=0.0)
    kept = set(np.nonzero(c.alpha)[0].tolist())
    assert kept == {1, 2, 4, 5, 6}
    assert c.alpha[4] == 2.0 and c.alpha[5] == -0.5 and c.alpha[6] == 1.0
    assert c.alpha[7] == 0.0                      # a zero row has zero residual: kept, with coefficient 0
    assert c.eta == 12 - 6
