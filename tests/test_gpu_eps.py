"""GPU parity for the neighbourhood condition (Eq. 2) and the normalisation factor beta (Sec. 3.2):
pamm_compress_eps / pamm_compress_idx_eps / pamm_grad_eps against the fp64 oracle, same seeded inputs.

Bars: f as in the unconditioned path; the kept/dropped decision equal for every row whose oracle residual is not
within 1e-6 ||X_i|| of the limit eps ||X_i|| (the decision is taken in fp64 on both sides, from different but
equivalent formulas); eta consistent with the GPU's own decisions and equal to the oracle's when no row sits in
that band; alpha and dW within the bars of the unconditioned path.
"""
import numpy as np
import pytest
import torch

from paper_2506_02939_amd import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TOL_ALPHA = 2e-5
TOL_DW = {"f32": 2e-5, "bf16": 2.0 ** -8}


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


def run_eps_case(pamm, oracle, X, dY, k, dtype_name, eps, *, seed=0, idx=None, label=""):
    b = X.shape[0]
    print(f"[case] {label} b={b} n={X.shape[1]} m={dY.shape[1]} k={k} {dtype_name} eps={eps}", flush=True)
    Xg, dYg = X.cuda(), dY.cuda()
    if idx is None:
        ora = oracle.compress(X, k, seed=seed, eps=eps)
        free = oracle.compress(X, k, seed=seed)
        got = pamm.compress(Xg, k, seed=seed, eps=eps)
    else:
        ia = np.asarray(idx, dtype=np.int32)
        ora = oracle.compress(X, k, idx=ia, eps=eps)
        free = oracle.compress(X, k, idx=ia)
        got = pamm.compress(Xg, k, idx=torch.as_tensor(ia).cuda(), eps=eps)
    torch.cuda.synchronize()
    f_gpu = got.f.cpu().numpy()
    a_gpu = got.alpha.cpu().numpy().astype(np.float64)
    eta_gpu = int(got.eta.cpu().item())
    assert np.isfinite(a_gpu).all() and 0 <= eta_gpu < b

    # assignment: as in the unconditioned path (dropped rows keep their f)
    gap = np.where(ora.best > 0, (ora.best - ora.second) / np.where(ora.best > 0, ora.best, 1.0), 0.0)
    near = gap < 1e-6
    assert np.array_equal(f_gpu[~near], ora.f[~near])
    agree = f_gpu == ora.f

    # kept / dropped
    margin = ora.resid - eps * ora.rownorm
    band = (np.abs(margin) <= 1e-6 * ora.rownorm) & (ora.resid > 0)
    live = free.alpha != 0                       # rows whose coefficient is not zero to begin with
    kept_or = ora.alpha != 0
    kept_gpu = a_gpu != 0
    check = agree & live & ~band
    assert np.array_equal(kept_gpu[check], kept_or[check]), f"{int(np.sum(kept_gpu[check] != kept_or[check]))} rows decided differently"
    # eta counts the rows the condition dropped.  A row whose coefficient is zero to begin with (a zero row, a row
    # orthogonal to its generator) is dropped or kept like any other without showing in alpha: those are counted
    # from the oracle's margin.
    if not band.any() and agree.all():
        assert eta_gpu == int(np.sum(~kept_gpu & live)) + int(np.sum(~live & (margin > 0)))
        assert eta_gpu == ora.eta
    e_alpha = rel_fro(a_gpu[check & kept_or], ora.alpha[check & kept_or]) if (check & kept_or).any() else 0.0
    assert e_alpha <= TOL[dtype_name] and e_alpha <= TOL_ALPHA, f"alpha error {e_alpha}"

    # ApproxMM with beta, on the GPU's own outputs: the oracle evaluated on the same (f, alpha, eta)
    beta_gpu = b / (b - eta_gpu)
    _, O_same = oracle.grad(ora.C, f_gpu, a_gpu, dY, beta=beta_gpu)
    dW = pamm.grad(got.C, got.f, got.alpha, dYg, eta=got.eta)
    torch.cuda.synchronize()
    e_dw = rel_fro(dW.cpu().numpy(), O_same)
    assert e_dw <= TOL[dtype_name] and e_dw <= TOL_DW[dtype_name], f"dW error {e_dw}"
    # ... and fed with the oracle's (f, alpha, eta)
    _, O_or = oracle.grad(ora.C, ora.f, ora.alpha, dY, beta=ora.beta)
    eta_in = torch.tensor([ora.eta], dtype=torch.int32).cuda()
    dW2 = pamm.grad(got.C, torch.from_numpy(ora.f).cuda(), torch.from_numpy(ora.alpha.astype(np.float32)).cuda(), dYg, eta=eta_in)
    torch.cuda.synchronize()
    e_dw2 = rel_fro(dW2.cpu().numpy(), O_or)
    assert e_dw2 <= TOL[dtype_name] and e_dw2 <= TOL_DW[dtype_name], f"dW (oracle f, alpha, eta) error {e_dw2}"
    print(f"[ok]   {label}: eta {eta_gpu} (oracle {ora.eta}, band rows {int(band.sum())}), alpha {e_alpha:.2e}, dW {e_dw:.2e} / {e_dw2:.2e}",
          flush=True)
    return ora, got


CASES = [
    # name, base workload, overrides
    ("f32_ragged", "tiny", dict(seqs=3, seq_len=171, n=100, m=524, k=5, centres=12)),
    ("bf16_k70", "llama60m", dict(seqs=4, seq_len=200, n=200, m=1032, k=70, centres=64)),
    ("bf16_k300_two_blocks", "llama7b_k256", dict(seqs=2, seq_len=700, n=136, m=264, k=300, centres=100)),
    ("bf16_ar1", "llama350m", dict(seqs=4, seq_len=128, n=256, m=768, k=16, centres=32)),
]


@pytest.mark.parametrize("eps", [0.0, 0.1, 0.35, 0.8])
@pytest.mark.parametrize("name,base,over", CASES, ids=[c[0] for c in CASES])
def test_small_shapes_with_tolerance(pamm, oracle, name, base, over, eps):
    w = workloads.scaled(workloads.WORKLOADS[base], name=name, **over)
    X, dY = workloads.generate(w)
    run_eps_case(pamm, oracle, X, dY, w.k, w.dtype, eps, seed=0, label=name)


def test_a_tolerance_of_one_or_more_drops_nothing(pamm, oracle):
    w = workloads.scaled(workloads.WORKLOADS["llama60m"], name="eps_ge_1", seqs=3, seq_len=150, n=128, m=136, k=9, centres=20)
    X, dY = workloads.generate(w)
    base = pamm.compress(X.cuda(), w.k, seed=4)
    for eps in (1.0, 7.5, float("inf")):
        got = pamm.compress(X.cuda(), w.k, seed=4, eps=eps)
        torch.cuda.synchronize()
        assert int(got.eta.cpu().item()) == 0
        assert torch.equal(got.f, base.f) and torch.equal(got.alpha, base.alpha)
        dW = pamm.grad(got.C, got.f, got.alpha, dY.cuda(), eta=got.eta)
        dW0 = pamm.grad(base.C, base.f, base.alpha, dY.cuda())
        torch.cuda.synchronize()
        assert torch.equal(dW, dW0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_zero_tolerance_keeps_exactly_the_collinear_rows(pamm, oracle, dtype):
    """eps = 0 is uniform column-row sampling: exact copies and power-of-two multiples of a generator survive (their
    residual is exactly zero), everything else is dropped, beta = b / kept."""
    g = torch.Generator().manual_seed(21)
    b, n, m = 700, 192, 136
    X = torch.randn(b, n, generator=g)
    X[10] = X[3]
    X[11] = -4.0 * X[3]
    X[12] = 0.5 * X[7]
    X[600:650] = X[7]
    X[20] = 0.0
    X = X.to(dtype)
    dY = (0.1 * torch.randn(b, m, generator=g)).to(dtype)
    idx = [3, 7, 100, 333]
    name = "f32" if dtype == torch.float32 else "bf16"
    ora, got = run_eps_case(pamm, oracle, X, dY, len(idx), name, 0.0, idx=idx, label=f"collinear {name}")
    a = got.alpha.cpu().numpy()
    kept = set(np.nonzero(a)[0].tolist())
    assert kept == {3, 7, 100, 333, 10, 11, 12} | set(range(600, 650))
    assert a[11] == -4.0 and a[12] == 0.5 and a[10] == 1.0
    assert int(got.eta.cpu().item()) == ora.eta == b - len(kept) - 1        # the zero row is kept with coefficient 0


def test_baseline_shape_with_tolerance(pamm, oracle):
    """The LLaMA-60M-shaped layer at full size with a tolerance that drops part of the batch."""
    w = workloads.WORKLOADS["llama60m"]
    X, dY = workloads.generate(w)
    ora, got = run_eps_case(pamm, oracle, X, dY, w.k, w.dtype, 0.25, seed=0, label="llama60m eps=0.25")
    assert 0 < ora.eta < w.b
