"""GPU test of the linear layer of Alg. 2 / Alg. 3 (paper_2506_02939_amd/linear.py): the weight gradient that autograd
returns is ApproxMM's estimate (checked against the fp64 oracle on the same inputs and seed), the input gradient and
the output are the exact products, and the backward pass keeps k n + 2 b numbers of X, not b n.
"""
import numpy as np
import pytest
import torch

from paper_2506_02939_amd import workloads

pytestmark = pytest.mark.gpu

TOL_DW = {"f32": 2e-5, "bf16": 2.0 ** -8}
ROUND16 = 2.0 ** -9


@pytest.fixture(scope="module")
def linear():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2506_02939_amd import linear as lin

    return lin


def rel_fro(a, ref):
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(a - ref) / den) if den > 0 else float(np.linalg.norm(a))


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


@pytest.mark.parametrize("base,out_by_in,eps", [("llama60m", False, None), ("llama60m", True, None), ("tiny", False, None),
                                                 ("llama60m", True, 0.3)],
                         ids=["bf16_n_by_m", "bf16_out_by_in", "f32_n_by_m", "bf16_out_by_in_eps"])
def test_backward_returns_the_approximate_weight_gradient(linear, oracle, base, out_by_in, eps):
    w = workloads.scaled(workloads.WORKLOADS[base], seqs=4, seq_len=96, n=136, m=264, centres=12)
    X2, dZ2 = workloads.generate(w)
    dn = "bf16" if X2.dtype == torch.bfloat16 else "f32"
    B, L, n, m = w.seqs, w.seq_len, w.n, w.m
    r, seed = 1.0 / 32, 9
    k = linear.generators_for(B * L, r)
    assert k == 12
    print(f"[case] linear layer b={B * L} n={n} m={m} k={k} {dn} out_by_in={out_by_in} eps={eps}", flush=True)
    g = torch.Generator().manual_seed(3)
    W = (torch.randn(n, m, generator=g) / n ** 0.5).to(X2.dtype)

    X = X2.view(B, L, n).cuda().requires_grad_(True)
    Wg = (W.t().contiguous() if out_by_in else W).cuda().requires_grad_(True)
    Z = linear.pamm_linear(X, Wg, r=r, seed=seed, eps=eps, out_by_in=out_by_in)
    saved = Z.grad_fn.saved_tensors
    Z.backward(dZ2.view(B, L, m).cuda())
    torch.cuda.synchronize()

    # what the backward pass kept of X: C (k x n), f and alpha (b each), besides W and, with eps, one counter
    kept = sum(t.numel() for t in saved if t.data_ptr() != Wg.data_ptr())
    assert kept <= k * n + 2 * B * L + 1 < B * L * n

    Xd, Wd = X.detach(), Wg.detach()
    assert torch.equal(Z.detach(), torch.matmul(Xd, Wd.t() if out_by_in else Wd))
    assert torch.equal(X.grad, torch.matmul(dZ2.view(B, L, m).cuda(), Wd if out_by_in else Wd.t()))

    ora = oracle.compress(X2, k, seed=seed, eps=float("inf") if eps is None else eps)
    _, O = oracle.grad(ora.C, ora.f, ora.alpha, dZ2, beta=ora.beta)
    assert Wg.grad.shape == Wg.shape and Wg.grad.dtype == Wg.dtype
    got = f64(Wg.grad.t() if out_by_in else Wg.grad)
    bar = TOL_DW[dn] + (ROUND16 if dn == "bf16" else 0.0)
    e = rel_fro(got, O)
    assert e <= bar, f"weight gradient error {e}"
    print(f"[ok]   linear layer: dW {e:.2e}", flush=True)


def test_layer_without_weight_gradient(linear):
    """Frozen weight (the LoRA setting of Sec. 4.7 freezes W0): only the exact input gradient is produced."""
    X = torch.randn(2, 64, 128, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    W = torch.randn(128, 136, device="cuda", dtype=torch.bfloat16)
    Z = linear.pamm_linear(X, W, k=2, seed=1)
    dZ = torch.randn_like(Z)
    Z.backward(dZ)
    torch.cuda.synchronize()
    assert torch.equal(X.grad, torch.matmul(dZ, W.t()))


@pytest.mark.parametrize("out_by_in,eps", [(False, None), (True, 0.3)])
def test_overlapped_layer_gives_the_same_bits(linear, out_by_in, eps):
    """overlap=True moves Compress and ApproxMM to a second stream beside the exact GEMMs: output and both gradients must
    be bit for bit those of the layer run on one stream, step after step (the streams are joined before each pass returns)."""
    w = workloads.scaled(workloads.WORKLOADS["llama350m"], seqs=4, seq_len=512, n=256, m=776, centres=40)
    X2, dZ2 = workloads.generate(w)
    g = torch.Generator().manual_seed(5)
    W0 = (torch.randn(w.n, w.m, generator=g) / w.n ** 0.5).to(X2.dtype)
    W0 = (W0.t().contiguous() if out_by_in else W0).cuda()
    res = []
    for overlap in (False, True, True):
        X = X2.view(w.seqs, w.seq_len, w.n).cuda().requires_grad_(True)
        Wg = W0.clone().requires_grad_(True)
        Z = linear.pamm_linear(X, Wg, k=24, seed=11, eps=eps, out_by_in=out_by_in, overlap=overlap)
        Z.backward(dZ2.view(w.seqs, w.seq_len, w.m).cuda())
        torch.cuda.synchronize()
        res.append((Z.detach().clone(), X.grad.clone(), Wg.grad.clone()))
    for other in res[1:]:
        assert all(torch.equal(a, b) for a, b in zip(res[0], other))
