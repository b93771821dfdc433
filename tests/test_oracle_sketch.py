"""Pins for the oracle's random-projection baseline (Sec. 4.6: the layer keeps S = A P and estimates the weight
gradient as P S^T B).  Every expected value is written out in numpy from the definition or is a closed form; shapes
are non-square (b != n != r != m) so that a transposed operand or a swapped index cannot pass.  Nothing here runs on
the GPU.
"""
import numpy as np
import torch


def _rng(seed):
    return np.random.default_rng(seed)


def _bf16_bits(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_identity_projection_keeps_everything(oracle):
    """r = n, P = I: the sketch is the input itself and the estimate is the exact product A^T B."""
    g = _rng(1)
    b, n, m = 23, 7, 5
    A, B = g.standard_normal((b, n)), g.standard_normal((b, m))
    S = oracle.sketch(A, np.eye(n))
    assert np.array_equal(S, A)
    G, O = oracle.sketch_grad(np.eye(n), S, B)
    assert np.allclose(G, A.T @ B, rtol=1e-13, atol=1e-13)
    assert np.allclose(O, A.T @ B, rtol=1e-13, atol=1e-13)


def test_orthogonal_projection_gives_the_exact_product(oracle):
    """Any orthogonal P has P P^T = I: the estimate (P P^T) A^T B is exact.  Q is not symmetric, so taking P for its
    transpose anywhere (in the sketch or in the last product) would change S or O."""
    g = _rng(2)
    b, n, m = 31, 9, 4
    A, B = g.standard_normal((b, n)), g.standard_normal((b, m))
    Q, _ = np.linalg.qr(g.standard_normal((n, n)))
    P = Q                                   # n x n
    S = oracle.sketch(A, P.T.copy())
    assert np.allclose(S, A @ P, rtol=1e-12, atol=1e-12)
    assert not np.allclose(S, A @ P.T, rtol=1e-3, atol=1e-3)
    G, O = oracle.sketch_grad(P.T.copy(), S, B)
    assert np.allclose(G, (A @ P).T @ B, rtol=1e-12, atol=1e-12)
    assert np.allclose(O, A.T @ B, rtol=1e-11, atol=1e-11)


def test_coordinate_selection(oracle):
    """P made of columns of the identity: the sketch keeps those coordinates of every row, and the estimate is the
    exact product on the kept coordinates and zero on the others."""
    g = _rng(3)
    b, n, m = 17, 10, 6
    sel = np.array([7, 2, 5])
    A, B = g.standard_normal((b, n)), g.standard_normal((b, m))
    Pt = np.zeros((len(sel), n))
    Pt[np.arange(len(sel)), sel] = 1.0
    S = oracle.sketch(A, Pt)
    assert np.array_equal(S, A[:, sel])
    G, O = oracle.sketch_grad(Pt, S, B)
    exact = A.T @ B
    want = np.zeros_like(exact)
    want[sel] = exact[sel]
    assert np.allclose(G, exact[sel], rtol=1e-13, atol=1e-13)
    assert np.allclose(O, want, rtol=1e-13, atol=1e-13)


def test_rank_one_closed_form(oracle):
    """r = 1, P = p: the estimate is p p^T A^T B."""
    g = _rng(4)
    b, n, m = 19, 6, 8
    A, B, p = g.standard_normal((b, n)), g.standard_normal((b, m)), g.standard_normal(n)
    S = oracle.sketch(A, p[None, :])
    assert np.allclose(S[:, 0], A @ p, rtol=1e-13, atol=1e-13)
    _, O = oracle.sketch_grad(p[None, :], S, B)
    assert np.allclose(O, np.outer(p, p) @ (A.T @ B), rtol=1e-12, atol=1e-12)


def test_gaussian_projection_is_unbiased(oracle):
    """Entries of P drawn from N(0, 1/r) give E[P P^T] = I: the mean of the estimate over many draws approaches
    A^T B at the rate 1/sqrt(draws).  (With entries N(0, 1/n) it would approach (r/n) A^T B instead.)"""
    g = _rng(5)
    b, n, m, r, draws = 8, 6, 3, 2, 6000
    A, B = g.standard_normal((b, n)), g.standard_normal((b, m))
    exact = A.T @ B
    mean = np.zeros_like(exact)
    for _ in range(draws):
        Pt = g.standard_normal((r, n)) / np.sqrt(r)
        mean += oracle.sketch_grad(Pt, oracle.sketch(A, Pt), B)[1]
    mean /= draws
    err = np.linalg.norm(mean - exact) / np.linalg.norm(exact)
    assert err < 0.08, err                                   # one standard error is about 0.03 here
    assert np.linalg.norm(mean - (r / n) * exact) / np.linalg.norm(exact) > 0.4


def test_linear_in_both_inputs_and_additive_over_rows(oracle):
    g = _rng(6)
    b, n, m, r = 14, 8, 5, 3
    A, B = g.standard_normal((b, n)), g.standard_normal((b, m))
    Pt = g.standard_normal((r, n))
    S = oracle.sketch(A, Pt)
    _, O = oracle.sketch_grad(Pt, S, B)
    _, O2 = oracle.sketch_grad(Pt, oracle.sketch(2.0 * A, Pt), -3.0 * B)
    assert np.allclose(O2, -6.0 * O, rtol=1e-12, atol=1e-12)
    _, Oa = oracle.sketch_grad(Pt, S[:5], B[:5])
    _, Ob = oracle.sketch_grad(Pt, S[5:], B[5:])
    assert np.allclose(Oa + Ob, O, rtol=1e-12, atol=1e-12)


def test_element_types_decode_to_the_same_values(oracle):
    """bfloat16 and float32 inputs holding the same values give the same sketch and estimate as float64 ones; the stored
    sketch is taken in its own element type."""
    g = _rng(7)
    b, n, m, r = 12, 8, 6, 4
    A16, B16, P16 = _bf16_bits(g.standard_normal((b, n))), _bf16_bits(g.standard_normal((b, m))), _bf16_bits(g.standard_normal((r, n)))
    A, B, Pt = oracle.to_f64(A16), oracle.to_f64(B16), oracle.to_f64(P16)
    S = oracle.sketch(A16, P16)
    assert np.array_equal(S, oracle.sketch(A, Pt))
    assert np.array_equal(S, oracle.sketch(A.astype(np.float32), Pt.astype(np.float32)))
    S16 = _bf16_bits(S)
    G, O = oracle.sketch_grad(P16, S16, B16)
    G2, O2 = oracle.sketch_grad(Pt, oracle.to_f64(S16), B)
    assert np.array_equal(G, G2) and np.array_equal(O, O2)
    assert np.allclose(G, oracle.to_f64(S16).T @ B, rtol=1e-13, atol=1e-13)
