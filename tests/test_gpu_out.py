"""GPU parity for pamm_grad_out (element type and orientation of the weight gradient) and for the shapes of the
fine-tuning settings (Sec. 4.1: down to a single generator; Sec. 4.3: batches of a few dozen to a few thousand
tokens; App. J's example works per projection, m = n).

Bars: the unconditioned path's (f outside near-ties, alpha and dW in relative Frobenius norm against the fp64
oracle).  A bf16 result carries one more rounding to nearest even of every element (relative error <= 2^-9 each),
so its bar is the fp32 result's plus 2^-9; two exact statements are checked besides: the m x n result is the
transpose of the n x m result bit for bit, and the bf16 result is the fp32 result rounded to nearest even.
"""
import numpy as np
import pytest
import torch

from paper_2506_02939_amd import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TOL_ALPHA = 2e-5
TOL_DW = {"f32": 2e-5, "bf16": 2.0 ** -8}
ROUND16 = 2.0 ** -9


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


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


SHAPES = [
    # name, base workload, overrides
    ("f32_ragged", "tiny", dict(seqs=3, seq_len=171, n=100, m=524, k=5, centres=12)),
    ("f32_two_tiles", "tiny", dict(seqs=2, seq_len=300, n=260, m=136, k=33, centres=40)),
    ("bf16_ragged", "llama60m", dict(seqs=5, seq_len=77, n=72, m=520, k=7, centres=16)),
    ("bf16_k70", "llama60m", dict(seqs=4, seq_len=200, n=200, m=1032, k=70, centres=64)),
    ("bf16_square", "llama350m", dict(seqs=2, seq_len=256, n=384, m=384, k=20, centres=32)),
]


@pytest.mark.parametrize("name,base,over", SHAPES, ids=[s[0] for s in SHAPES])
def test_element_type_and_orientation_of_dw(pamm, oracle, name, base, over):
    w = workloads.scaled(workloads.WORKLOADS[base], **over)
    X, dY = workloads.generate(w)
    dn = "bf16" if X.dtype == torch.bfloat16 else "f32"
    print(f"[case] out {name} b={w.b} n={w.n} m={w.m} k={w.k} {dn}", flush=True)
    ora = oracle.compress(X, w.k, seed=3)
    _, O = oracle.grad(ora.C, ora.f, ora.alpha, dY)
    Cg = torch.as_tensor(np.ascontiguousarray(X.view(torch.int16 if dn == "bf16" else torch.int32).numpy()[ora.idx])).view(X.dtype).cuda()
    fg = torch.from_numpy(ora.f).cuda()
    ag = torch.from_numpy(ora.alpha.astype(np.float32)).cuda()
    dYg = dY.cuda()

    base32 = pamm.grad(Cg, fg, ag, dYg)
    same32 = pamm.grad(Cg, fg, ag, dYg, out_dtype=torch.float32)
    t32 = pamm.grad(Cg, fg, ag, dYg, transposed=True)
    o16 = pamm.grad(Cg, fg, ag, dYg, out_dtype=torch.bfloat16)
    t16 = pamm.grad(Cg, fg, ag, dYg, out_dtype=torch.bfloat16, transposed=True)
    torch.cuda.synchronize()
    assert t32.shape == (w.m, w.n) and o16.shape == (w.n, w.m) and t16.shape == (w.m, w.n)
    assert o16.dtype == torch.bfloat16 and t16.dtype == torch.bfloat16

    e32 = rel_fro(f64(base32), O)
    assert e32 <= TOL[dn] and e32 <= TOL_DW[dn]
    assert torch.equal(same32, base32), "pamm_grad_out(fp32, n x m) differs from pamm_grad"
    assert torch.equal(t32.t().contiguous(), base32), "the m x n result is not the transpose of the n x m result"
    assert torch.equal(o16, base32.to(torch.bfloat16)), "the bf16 result is not the fp32 result rounded to nearest even"
    assert torch.equal(t16.t().contiguous(), o16)
    for got in (o16, t16.t()):
        e = rel_fro(f64(got), O)
        assert e <= TOL_DW[dn] + ROUND16 and e <= max(TOL[dn], ROUND16 + TOL_DW[dn]), f"bf16 dW error {e}"
    print(f"[ok]   out {name}: dW fp32 {e32:.2e}, bf16 {rel_fro(f64(o16), O):.2e}", flush=True)


def test_orientation_and_type_with_beta(pamm, oracle):
    """The normalisation factor of Sec. 3.2 goes through pamm_grad_out like through pamm_grad_eps."""
    w = workloads.scaled(workloads.WORKLOADS["llama60m"], seqs=4, seq_len=128, n=136, m=264, k=24, centres=24)
    X, dY = workloads.generate(w)
    print(f"[case] out with beta b={w.b} n={w.n} m={w.m} k={w.k}", flush=True)
    ora = oracle.compress(X, w.k, seed=1, eps=0.3)
    assert 0 < ora.eta < w.b
    _, O = oracle.grad(ora.C, ora.f, ora.alpha, dY, beta=ora.beta)
    got = pamm.compress(X.cuda(), w.k, seed=1, eps=0.3)
    ref = pamm.grad(got.C, got.f, got.alpha, dY.cuda(), eta=got.eta)
    t16 = pamm.grad(got.C, got.f, got.alpha, dY.cuda(), eta=got.eta, out_dtype=torch.bfloat16, transposed=True)
    torch.cuda.synchronize()
    assert int(got.eta.item()) == ora.eta
    assert torch.equal(t16.t().contiguous(), ref.to(torch.bfloat16))
    assert rel_fro(f64(t16.t()), O) <= TOL_DW["bf16"] + ROUND16


FINE_TUNING = [
    # name, dtype base, b = seqs x seq_len, n, m, k
    ("k1_b64", "llama60m", 1, 64, 256, 256, 1),
    ("k1_b1000", "llama60m", 4, 250, 512, 512, 1),
    ("k2_b136", "llama60m", 1, 136, 768, 2304, 2),
    ("k4_b2048", "llama60m", 8, 256, 768, 768, 4),
    ("k4_b8192_per_projection", "llama350m", 16, 512, 1024, 1024, 4),
    ("k1_b8_f32", "tiny", 1, 8, 64, 64, 1),
    ("k2_b100_f32", "tiny", 1, 100, 128, 384, 2),
    ("k4_b4096_f32", "tiny", 16, 256, 256, 256, 4),
]


@pytest.mark.parametrize("name,base,seqs,seq_len,n,m,k", FINE_TUNING, ids=[s[0] for s in FINE_TUNING])
def test_fine_tuning_shapes(pamm, oracle, name, base, seqs, seq_len, n, m, k):
    w = workloads.scaled(workloads.WORKLOADS[base], seqs=seqs, seq_len=seq_len, n=n, m=m, k=k, centres=8)
    X, dY = workloads.generate(w)
    dn = "bf16" if X.dtype == torch.bfloat16 else "f32"
    print(f"[case] fine-tuning {name} b={w.b} n={n} m={m} k={k} {dn}", flush=True)
    ora = oracle.compress(X, k, seed=5)
    _, O = oracle.grad(ora.C, ora.f, ora.alpha, dY)
    got = pamm.compress(X.cuda(), k, seed=5)
    dW = pamm.grad(got.C, got.f, got.alpha, dY.cuda())
    dWt = pamm.grad(got.C, got.f, got.alpha, dY.cuda(), out_dtype=X.dtype, transposed=True)
    torch.cuda.synchronize()
    f_gpu = got.f.cpu().numpy()
    gap = np.where(ora.best > 0, (ora.best - ora.second) / np.where(ora.best > 0, ora.best, 1.0), 0.0)
    near = gap < 1e-6
    assert np.array_equal(f_gpu[~near], ora.f[~near])
    agree = f_gpu == ora.f
    e_alpha = rel_fro(got.alpha.cpu().numpy()[agree], ora.alpha[agree])
    assert e_alpha <= TOL_ALPHA
    if not agree.all():
        _, O = oracle.grad(ora.C, f_gpu, got.alpha.cpu().numpy().astype(np.float64), dY)
    e = rel_fro(f64(dW), O)
    assert e <= TOL[dn] and e <= TOL_DW[dn], f"dW error {e}"
    assert torch.equal(dWt.t().contiguous(), dW.to(X.dtype))
    if k == 1:
        # a single generator: dW is the outer product of C_1 with alpha^T dY (Sec. 4.1)
        v = (got.alpha.cpu().to(torch.float64)[:, None] * dY.to(torch.float64)).sum(0).numpy()
        outer = np.outer(f64(got.C)[0], v)
        assert rel_fro(f64(dW), outer) <= TOL_DW[dn]
    print(f"[ok]   fine-tuning {name}: alpha {e_alpha:.2e}, dW {e:.2e}", flush=True)


def test_argument_checks_of_grad_out(pamm):
    dev = torch.device("cuda")
    b, n, m, k = 64, 8, 12, 2
    C = torch.zeros(k, n, device=dev)
    f = torch.zeros(b, dtype=torch.int32, device=dev)
    a = torch.ones(b, device=dev)
    dY = torch.zeros(b, m, device=dev)
    ws = torch.empty(pamm.grad_workspace(b, n, k, m, pamm.PAMM_F32), dtype=torch.uint8, device=dev)
    out = torch.full((n, m), 7.0, device=dev)

    def call(out_dt, layout):
        return pamm.lib.pamm_grad_out(C.data_ptr(), f.data_ptr(), a.data_ptr(), None, dY.data_ptr(), b, n, k, m, pamm.PAMM_F32,
                                      out_dt, layout, out.data_ptr(), ws.data_ptr(), ws.numel(), None)

    assert call(5, pamm.PAMM_DW_N_BY_M) == pamm.PAMM_ERR_UNSUPPORTED
    assert call(pamm.PAMM_F32, 2) == pamm.PAMM_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((out == 7.0).all()), "a refused call touched its output"
    assert call(pamm.PAMM_F32, pamm.PAMM_DW_M_BY_N) == pamm.PAMM_OK
    torch.cuda.synchronize()
    assert bool((out == 0.0).all())
