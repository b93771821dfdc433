"""GPU parity on a seeded sweep of random small shapes: sizes that no hand-picked case has (odd token counts, row
lengths one chunk long, k from 1 to b, both element types, with and without the tolerance of Eq. 2), each run through
pamm_compress / pamm_grad (or their _eps / _out forms) and compared with the fp64 oracle at the bars of the other
parity tests.  The shapes are drawn from a fixed seed, so every run checks the same list.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

TOL_ALPHA = 2e-5
TOL_DW = {"f32": 2e-5, "bf16": 2.0 ** -8}
ROUND16 = 2.0 ** -9


def _shapes():
    g = np.random.default_rng(20250601)
    out = []
    for i in range(48):
        bf16 = bool(g.integers(0, 2))
        unit = 8 if bf16 else 4
        b = int(g.choice([1, 2, 3, 31, 33, 64, 100, 255, 257, 511, 1000, 1025, 2049, 3000, 4097, 9001]))
        n = unit * int(g.integers(1, 70))
        m = unit * int(g.integers(1, 70))
        kmax = min(b, 700)
        k = int(g.choice([1, 2, 3, 5, 16, 17, 31, 32, 33, 64, 100, 255, 256, 257, 300, 513, 700]))
        k = max(1, min(k, kmax))
        eps = [None, None, 0.0, 0.25, 0.6][int(g.integers(0, 5))]
        form = ["plain", "plain", "bf16", "t", "t_bf16"][int(g.integers(0, 5))]
        out.append((i, "bf16" if bf16 else "f32", b, n, m, k, eps, form))
    return out


SHAPES = _shapes()


@pytest.fixture(scope="module")
def pamm():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2506_02939_amd import pamm as p

    return p


def rel_fro(a, ref):
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(a - ref) / den) if den > 0 else float(np.linalg.norm(a))


@pytest.mark.parametrize("case", SHAPES, ids=[f"{c[0]:02d}_{c[1]}_b{c[2]}_n{c[3]}_m{c[4]}_k{c[5]}_eps{c[6]}_{c[7]}" for c in SHAPES])
def test_random_shape(pamm, oracle, case):
    i, dn, b, n, m, k, eps, form = case
    print(f"[case] random shape {case}", flush=True)
    g = torch.Generator().manual_seed(1000 + i)
    dt = torch.bfloat16 if dn == "bf16" else torch.float32
    centres = max(1, min(b, 2 * k))
    mu = torch.randn(centres, n, generator=g)
    z = torch.randint(0, centres, (b,), generator=g)
    s = torch.rand(b, generator=g) * 1.5 + 0.5
    X = (mu[z] * s[:, None] + 0.15 * torch.randn(b, n, generator=g)).to(dt)
    if b >= 4:
        X[b // 2] = X[0]                       # an exact duplicate and a zero row in every batch that has room
        X[b - 1] = 0
    dY = (0.1 * torch.randn(b, m, generator=g)).to(dt)

    ora = oracle.compress(X, k, seed=i, eps=float("inf") if eps is None else eps)
    got = pamm.compress(X.cuda(), k, seed=i, eps=eps)
    torch.cuda.synchronize()
    f_gpu = got.f.cpu().numpy()
    a_gpu = got.alpha.cpu().numpy().astype(np.float64)
    assert np.isfinite(a_gpu).all() and f_gpu.min() >= 0 and f_gpu.max() < k

    gap = np.where(ora.best > 0, (ora.best - ora.second) / np.where(ora.best > 0, ora.best, 1.0), 0.0)
    near = gap < 1e-6
    assert np.array_equal(f_gpu[~near], ora.f[~near]), "assignment differs outside near-ties"
    # rows whose kept/dropped decision is not within 1e-6 ||X_i|| of the limit must agree on it
    sure = ~near
    if eps is not None:
        margin = np.abs(ora.resid - eps * ora.rownorm)
        sure &= margin > 1e-6 * np.maximum(ora.rownorm, 1e-300)
    assert np.array_equal((a_gpu != 0)[sure], (ora.alpha != 0)[sure]), "kept / dropped decision differs away from the limit"
    same = sure & (f_gpu == ora.f)
    assert rel_fro(a_gpu[same], ora.alpha[same]) <= TOL_ALPHA

    # ApproxMM on the GPU's own (f, alpha): the oracle recomputes from exactly those
    eta_gpu = int(got.eta.item()) if got.eta is not None else 0
    beta = (b / (b - eta_gpu)) if eta_gpu < b else 0.0
    _, O = oracle.grad(ora.C, f_gpu, a_gpu, dY, beta=beta if eps is not None else 1.0)
    kw = {}
    if form in ("bf16", "t_bf16"):
        kw["out_dtype"] = torch.bfloat16
    if form in ("t", "t_bf16"):
        kw["transposed"] = True
    dW = pamm.grad(got.C, got.f, got.alpha, dY.cuda(), eta=got.eta, **kw)
    torch.cuda.synchronize()
    dWn = dW.t() if "transposed" in kw else dW
    e = rel_fro(dWn.cpu().to(torch.float64).numpy(), O)
    bar = TOL_DW[dn] + (ROUND16 if "out_dtype" in kw else 0.0)
    assert e <= bar, f"dW error {e} > {bar}"
    print(f"[ok]   random shape {i}: dW {e:.2e}", flush=True)
