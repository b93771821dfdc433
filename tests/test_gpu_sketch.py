"""GPU parity of the random-projection baseline (Sec. 4.6: the layer keeps S = X P and estimates the weight gradient as
P S^T dY) against the fp64 oracle, element by element.

Bars (u = 2^-8, the unit roundoff of bf16; abs(.) marks the same expression evaluated on absolute values, the
scale that rounding errors are relative to):
  S     bf16: u |S| + 6e-6 abs(S)   one rounding of the stored sketch on top of an fp32 sum of exact products
        f32 : 1e-5 abs(S)            fp32 products and sums
  dW    bf16: (u + 5e-6) abs(dW)    G = S^T dY summed in fp32, rounded once to bf16, times Pt^T in fp32: the bar of
                                    pamm_grad's bf16 path, whose last two steps these are
        f32 : 5e-6 abs(dW)          nothing is rounded to 16 bits: pamm_grad's fp32 bar
"""
import numpy as np
import pytest
import torch

from paper_2506_02939_amd import workloads

pytestmark = pytest.mark.gpu

U16 = 2.0 ** -8


@pytest.fixture(scope="module")
def pamm():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2506_02939_amd import pamm as p

    return p


def _check_sketch(oracle, X, Pt, S_gpu):
    S = oracle.sketch(X, Pt)
    S_abs = oracle.sketch(X.abs(), Pt.abs())
    got = S_gpu.float().cpu().numpy().astype(np.float64)
    if X.dtype == torch.bfloat16:
        bar = (U16 + 1e-6) * np.abs(S) + 6e-6 * S_abs
    else:
        bar = 1e-5 * S_abs
    err = np.abs(got - S)
    assert np.all(err <= bar + 1e-30), f"S off by {np.max(err / np.maximum(bar, 1e-300))} bars"


def _check_grad(oracle, Pt, S, dY, dW_gpu):
    _, O = oracle.sketch_grad(Pt, S, dY)
    _, O_abs = oracle.sketch_grad(Pt.abs(), S.abs(), dY.abs())
    err = np.abs(dW_gpu.cpu().numpy().astype(np.float64) - O)
    u = U16 if dY.dtype == torch.bfloat16 else 0.0
    assert np.all(err <= (u + 5e-6) * O_abs + 1e-30), f"dW off by {np.max(err / np.maximum(O_abs, 1e-300))}"
    assert np.linalg.norm(err) <= (u + 2e-5) * np.linalg.norm(O)


CASES = [
    # name, base workload, overrides, sketch width
    ("r8_ragged", "llama60m", dict(seqs=5, seq_len=77, n=72, m=520, k=7, centres=16), 8),
    ("r24_two_column_groups", "llama60m", dict(seqs=3, seq_len=333, n=200, m=1032, k=7, centres=16), 24),
    ("r40", "llama350m", dict(seqs=4, seq_len=300, n=264, m=776, k=7, centres=32), 40),
    ("r72", "llama350m", dict(seqs=2, seq_len=450, n=136, m=1544, k=7, centres=32), 72),
    ("r128_many_chunks", "llama1b", dict(seqs=9, seq_len=1000, n=256, m=2056, k=7, centres=64), 128),
    ("r16_many_chunks", "llama1b", dict(seqs=16, seq_len=1021, n=512, m=4608, k=7, centres=64), 16),
]


@pytest.mark.parametrize("name,base,over,r", CASES, ids=[c[0] for c in CASES])
def test_sketch_and_its_gradient_estimate(pamm, oracle, name, base, over, r):
    w = workloads.scaled(workloads.WORKLOADS[base], **over)
    X, dY = workloads.generate(w)
    Pt = workloads.sketch_directions(w, r)
    print(f"[case] sketch {name} b={w.b} n={w.n} m={w.m} r={r}", flush=True)
    S_gpu = pamm.sketch(X.cuda(), Pt.cuda())
    torch.cuda.synchronize()
    assert S_gpu.shape == (w.b, r) and S_gpu.dtype == X.dtype
    _check_sketch(oracle, X, Pt, S_gpu)
    # the estimate from the GPU's own sketch, and from the oracle's (rounded to the element type the layer keeps)
    dW = pamm.sketch_grad(Pt.cuda(), S_gpu, dY.cuda())
    dW2 = pamm.sketch_grad(Pt.cuda(), S_gpu, dY.cuda())
    torch.cuda.synchronize()
    assert dW.shape == (w.n, w.m) and dW.dtype == torch.float32
    assert torch.equal(dW, dW2), "two calls on the same inputs differ"
    _check_grad(oracle, Pt, S_gpu.cpu(), dY, dW)
    S_or = torch.from_numpy(oracle.sketch(X, Pt)).to(X.dtype)
    dW3 = pamm.sketch_grad(Pt.cuda(), S_or.cuda(), dY.cuda())
    torch.cuda.synchronize()
    _check_grad(oracle, Pt, S_or, dY, dW3)


def _random_shapes():
    g = np.random.default_rng(20250907)
    out = []
    for i in range(24):
        b = int(g.choice([8, 9, 31, 33, 100, 255, 257, 1000, 1025, 3000, 4097, 9001]))
        n = 8 * int(g.integers(1, 70))
        m = 8 * int(g.integers(1, 140))
        r = 8 * int(g.integers(1, 17))
        out.append((i, b, n, m, min(r, b // 8 * 8)))
    return out


RANDOM_SHAPES = _random_shapes()


@pytest.mark.parametrize("case", RANDOM_SHAPES, ids=[f"{c[0]:02d}_b{c[1]}_n{c[2]}_m{c[3]}_r{c[4]}" for c in RANDOM_SHAPES])
def test_random_shape(pamm, oracle, case):
    """A seeded sweep of small shapes no hand-picked case has: token counts that are no multiple of a stage, rows one
    chunk long, every sketch width from 8 to 128."""
    i, b, n, m, r = case
    print(f"[case] sketch random shape {case}", flush=True)
    g = torch.Generator().manual_seed(3000 + i)
    X = torch.randn(b, n, generator=g).to(torch.bfloat16)
    dY = (0.1 * torch.randn(b, m, generator=g)).to(torch.bfloat16)
    Pt = (torch.randn(r, n, generator=g) / r ** 0.5).to(torch.bfloat16)
    S = pamm.sketch(X.cuda(), Pt.cuda())
    dW = pamm.sketch_grad(Pt.cuda(), S, dY.cuda())
    torch.cuda.synchronize()
    assert torch.isfinite(dW).all()
    _check_sketch(oracle, X, Pt, S)
    _check_grad(oracle, Pt, S.cpu(), dY, dW)


@pytest.mark.parametrize("n,m,r", [(256, 64, 8), (100, 524, 20), (516, 1028, 128), (64, 260, 4), (136, 300, 68), (72, 2052, 36)])
def test_fp32_inputs(pamm, oracle, n, m, r):
    """fp32 elements: plain LDS reads feed the fp32 MFMA, nothing is rounded to 16 bits; every fragment count, sketch
    widths that are no multiple of 8, ragged edges."""
    w = workloads.scaled(workloads.WORKLOADS["tiny"], seqs=3, seq_len=571, n=n, m=m, k=5, centres=12)
    X, dY = workloads.generate(w)
    Pt = workloads.sketch_directions(w, r)
    S_gpu = pamm.sketch(X.cuda(), Pt.cuda())
    dW = pamm.sketch_grad(Pt.cuda(), S_gpu, dY.cuda())
    dW2 = pamm.sketch_grad(Pt.cuda(), S_gpu, dY.cuda())
    torch.cuda.synchronize()
    assert torch.equal(dW, dW2)
    _check_sketch(oracle, X, Pt, S_gpu)
    _check_grad(oracle, Pt, S_gpu.cpu(), dY, dW)


def test_identity_directions_reproduce_the_input_and_the_exact_product(pamm, oracle):
    """r = n = 128 with P = I: S is X bit for bit, and the estimate is X^T dY at the bar."""
    w = workloads.scaled(workloads.WORKLOADS["llama60m"], seqs=3, seq_len=250, n=128, m=520, k=7, centres=16)
    X, dY = workloads.generate(w)
    Pt = torch.eye(128, dtype=X.dtype)
    S = pamm.sketch(X.cuda(), Pt.cuda())
    torch.cuda.synchronize()
    assert torch.equal(S.cpu(), X)
    dW = pamm.sketch_grad(Pt.cuda(), S, dY.cuda())
    torch.cuda.synchronize()
    exact = oracle.to_f64(X).T @ oracle.to_f64(dY)
    exact_abs = np.abs(oracle.to_f64(X)).T @ np.abs(oracle.to_f64(dY))
    assert np.all(np.abs(dW.cpu().numpy().astype(np.float64) - exact) <= (U16 + 5e-6) * exact_abs)


@pytest.mark.parametrize("name,r", [("llama1b", 8), ("llama7b_k32", 16)])
def test_memory_matched_sketch_at_full_size(pamm, oracle, name, r):
    """The sketch as wide as PAMM's compression is big (b r >= k n + 2 b, a whole 16-byte row) at the 1B-shaped layer and
    at the 7B-shaped layer with 32 generators, full size, in the launch configuration the benchmark times; every element
    against the oracle."""
    w = workloads.WORKLOADS[name]
    assert workloads.matched_sketch_width(w) == r
    X, dY = workloads.generate(w)
    Pt = workloads.sketch_directions(w, r)
    S = pamm.sketch(X.cuda(), Pt.cuda())
    dW = pamm.sketch_grad(Pt.cuda(), S, dY.cuda())
    torch.cuda.synchronize()
    print(f"[case] sketch {name} r={r}: oracle", flush=True)
    _check_sketch(oracle, X, Pt, S)
    _check_grad(oracle, Pt, S.cpu(), dY, dW)


def test_sketch_step_can_be_captured_in_a_hip_graph(pamm):
    """pamm_sketch followed by pamm_sketch_grad allocate nothing, never synchronise and record no memset (the chunk of
    zeros is written by the kernel that reads it): every replay of a captured step, with eager work and synchronisations
    in between, must give the eager result bit for bit."""
    w = workloads.scaled(workloads.WORKLOADS["llama60m"], name="graph", seqs=4, seq_len=300, n=256, m=776, k=7, centres=40)
    X, dY = workloads.generate(w)
    X, dY = X.cuda(), dY.cuda()
    r = 24
    Pt = workloads.sketch_directions(w, r).cuda()
    S = torch.empty(w.b, r, dtype=X.dtype, device="cuda")
    dW = torch.empty(w.n, w.m, dtype=torch.float32, device="cuda")
    ws = torch.empty(pamm.sketch_grad_workspace(w.b, w.n, r, w.m, pamm.PAMM_BF16), dtype=torch.uint8, device="cuda")

    def step():
        pamm.sketch(X, Pt, out=S)
        pamm.sketch_grad(Pt, S, dY, out=dW, ws=ws)

    step()
    torch.cuda.synchronize()
    ref_s, ref_dw = S.clone(), dW.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for _ in range(4):
        S.zero_(); dW.zero_(); ws.fill_(0xff)
        junk = torch.randn(1 << 20, device="cuda").sum().item()       # eager work and a synchronisation between replays
        assert junk == junk
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(S, ref_s) and torch.equal(dW, ref_dw)


def test_argument_errors(pamm):
    from paper_2506_02939_amd.pamm import PammError, PAMM_ERR_UNSUPPORTED, PAMM_ERR_WORKSPACE, PAMM_ERR_INVALID_ARG, PAMM_BF16, PAMM_F32

    X = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda")
    dY = torch.zeros(256, 128, dtype=torch.bfloat16, device="cuda")
    for r in (12, 136):
        with pytest.raises(PammError) as e:
            pamm.sketch(X, torch.zeros(r, 64, dtype=torch.bfloat16, device="cuda"))
        assert e.value.status == PAMM_ERR_UNSUPPORTED
    Pt = torch.zeros(8, 64, dtype=torch.bfloat16, device="cuda")
    S = pamm.sketch(X, Pt)
    with pytest.raises(PammError) as e:
        pamm.sketch_grad(Pt, S, dY, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == PAMM_ERR_WORKSPACE
    assert pamm.sketch_grad_workspace(256, 64, 8, 128, PAMM_F32) > 0 and pamm.sketch_grad_workspace(256, 64, 8, 128, PAMM_BF16) > 0
    assert pamm.sketch_grad_workspace(256, 64, 8, 132, PAMM_BF16) == 0          # rows of dY not 16-byte aligned
    with pytest.raises(PammError) as e:          # more directions than rows
        pamm.sketch(X[:4], Pt)
    assert e.value.status == PAMM_ERR_INVALID_ARG
    torch.cuda.synchronize()
