"""pamm_grad_static, the entry point for callers that cannot allocate: through the C ABI, against pamm_grad on the same
inputs (same kernels, so bit for bit), on two calls in a row that share the library's static scratch array, the second
with a smaller input; and against the fp64 oracle at the bars of the other parity tests."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2506_02939_amd import workloads


@pytest.fixture(scope="module")
def pamm():
    from paper_2506_02939_amd import pamm as p

    return p


def test_sizes_beyond_the_static_array_are_refused_on_the_host(pamm):
    A = 0x10000
    call = lambda b, n, k, m: pamm.lib.pamm_grad_static(A, A, A, A, b, n, k, m, pamm.PAMM_BF16, A, None)
    assert pamm.grad_workspace(16384, 4096, 1024, 12288, pamm.PAMM_BF16) > pamm.STATIC_SCRATCH_BYTES
    assert call(16384, 4096, 1024, 12288) == pamm.PAMM_ERR_WORKSPACE
    assert pamm.grad_workspace(65536, 2048, 128, 6144, pamm.PAMM_BF16) <= pamm.STATIC_SCRATCH_BYTES
    assert call(64, 64, 65, 64) == pamm.PAMM_ERR_INVALID_ARG            # k > b
    assert call(64, 64, 4, 12) == pamm.PAMM_ERR_UNSUPPORTED
    assert pamm.lib.pamm_grad_static(None, A, A, A, 64, 64, 4, 64, pamm.PAMM_BF16, A, None) == pamm.PAMM_ERR_INVALID_ARG
    assert pamm.lib.pamm_grad_static(A, A, A, A, 64, 64, 4, 64, pamm.PAMM_BF16, None, None) == pamm.PAMM_ERR_INVALID_ARG


@pytest.mark.gpu
def test_static_scratch_gives_what_pamm_grad_gives_twice_in_a_row(pamm, oracle):
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    shapes = [
        dict(seqs=16, seq_len=1024, n=512, m=1544, k=70, centres=200),       # several chunks, a ragged column tail
        dict(seqs=3, seq_len=333, n=136, m=264, k=9, centres=20),            # smaller, right after: stale scratch around it
    ]
    for round_, over in enumerate(shapes):
        w = workloads.scaled(workloads.WORKLOADS["llama60m"], name=f"static{round_}", **over)
        X, dY = workloads.generate(w)
        print(f"[case] pamm_grad_static call {round_}: b={w.b} n={w.n} m={w.m} k={w.k}", flush=True)
        got = pamm.compress(X.cuda(), w.k, seed=round_)
        dYg = dY.cuda()
        ref = pamm.grad(got.C, got.f, got.alpha, dYg)
        out = torch.full((w.n, w.m), float("nan"), dtype=torch.float32, device="cuda")
        pamm.grad_static(got.C, got.f, got.alpha, dYg, out)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "pamm_grad_static differs from pamm_grad"
        fa = got.f.cpu().numpy()
        aa = got.alpha.cpu().numpy().astype(np.float64)
        _, O = oracle.grad(oracle.to_f64(got.C.cpu()), fa, aa, dY)
        _, O_abs = oracle.grad(np.abs(oracle.to_f64(got.C.cpu())), fa, np.abs(aa), dY.abs())
        err = np.abs(out.cpu().numpy().astype(np.float64) - O)
        assert np.linalg.norm(err) <= 2.0 ** -8 * np.linalg.norm(O)
        assert np.all(err <= (2.0 ** -8 + 5e-6) * O_abs)
