"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what include/pamm.h declares,
its sampler agrees with the oracle's, and every argument check fires before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pamm.h")


@pytest.fixture(scope="module")
def pamm():
    from paper_2506_02939_amd import pamm as p

    return p


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pamm_[a-z_]+)\s*\(", text)))


def test_header_and_library_agree(pamm):
    declared = _declared_functions()
    assert declared == sorted(pamm.EXPORTS)
    for name in declared:
        assert hasattr(pamm.lib, name), f"libpamm.so does not export {name}"


def test_status_strings(pamm):
    names = {pamm.status_string(i) for i in range(5)}
    assert names == {"PAMM_OK", "PAMM_ERR_INVALID_ARG", "PAMM_ERR_UNSUPPORTED", "PAMM_ERR_WORKSPACE", "PAMM_ERR_DEVICE"}
    assert pamm.status_string(99) == "PAMM_ERR_UNKNOWN"


@pytest.mark.parametrize("b,k,seed", [(10, 10, 0), (8192, 16, 0), (65536, 128, 0), (16384, 1024, 0), (16384, 32, 12345),
                                      (2048, 2048, 7), (3, 2, 2**64 - 1), (1, 1, 5)])
def test_sampler_matches_oracle_stream(pamm, oracle, b, k, seed):
    """Two independent implementations of the specified sampler (Alg. 1, 'sample indices'): same stream."""
    got = pamm.sample_indices(b, k, seed).numpy()
    assert np.array_equal(got, oracle.sample(b, k, seed))


def test_bounded_draw_hook_takes_the_rejection_branch_like_the_specification(pamm, oracle):
    """The library's bounded step on ranges near 2^63 (rejection probability 1/4 .. 1/2): against the published
    splitmix64 outputs reduced with exact integers, and draw for draw against the oracle's independent implementation."""
    golden = os.path.join(ROOT, "tests", "golden", "splitmix64_seed1234567.txt")
    pub = [int(line) for line in open(golden) if line.strip() and not line.startswith("#")]
    for u in (3 << 62, (1 << 63) + 12345, (1 << 62) + 1, 5):
        cut = (1 << 64) % u
        want = [x % u for x in pub if x >= cut]
        assert pamm.debug_bounded(1234567, u, len(want)) == want
        for seed in (0, 99, 2**64 - 1):
            assert pamm.debug_bounded(seed, u, 500) == [int(v) for v in oracle.bounded(seed, u, 500)]
    assert pamm.lib.pamm_debug_bounded(0, 0, 1, ctypes.addressof((ctypes.c_uint64 * 1)())) == pamm.PAMM_ERR_INVALID_ARG
    assert pamm.lib.pamm_debug_bounded(0, 5, 1, None) == pamm.PAMM_ERR_INVALID_ARG


def test_plan_overrides_enter_the_workspace_query_and_can_be_cleared(pamm):
    base = pamm.grad_workspace(65536, 2048, 128, 6144, pamm.PAMM_BF16)
    try:
        pamm.debug_set_plan(piece_rows=16)
        assert pamm.grad_workspace(65536, 2048, 128, 6144, pamm.PAMM_BF16) > base       # 4096 chunks of partial rows
        pamm.debug_set_plan(piece_rows=17)                                              # out of range: heuristic stays
        assert pamm.grad_workspace(65536, 2048, 128, 6144, pamm.PAMM_BF16) == base
        c0 = pamm.compress_workspace(16384, 4096, 1024, pamm.PAMM_BF16)
        pamm.debug_set_plan(score_tg=1)
        assert pamm.compress_workspace(16384, 4096, 1024, pamm.PAMM_BF16) > c0           # 32 column blocks of records
    finally:
        pamm.debug_set_plan()
    assert pamm.grad_workspace(65536, 2048, 128, 6144, pamm.PAMM_BF16) == base


def test_sampler_rejects_bad_arguments(pamm):
    buf = (ctypes.c_int32 * 4)()
    assert pamm.lib.pamm_sample_indices(4, 5, 0, ctypes.addressof(buf)) == pamm.PAMM_ERR_INVALID_ARG
    assert pamm.lib.pamm_sample_indices(4, 0, 0, ctypes.addressof(buf)) == pamm.PAMM_ERR_INVALID_ARG
    assert pamm.lib.pamm_sample_indices(0, 0, 0, ctypes.addressof(buf)) == pamm.PAMM_ERR_INVALID_ARG
    assert pamm.lib.pamm_sample_indices(4, 2, 0, None) == pamm.PAMM_ERR_INVALID_ARG


def test_workspace_queries(pamm):
    assert pamm.compress_workspace(65536, 2048, 128, pamm.PAMM_BF16) >= 65536 * 32
    assert pamm.grad_workspace(65536, 2048, 128, 6144, pamm.PAMM_BF16) >= 128 * 6144 * 4
    # invalid sizes -> 0
    assert pamm.compress_workspace(16, 64, 17, pamm.PAMM_BF16) == 0        # k > b
    assert pamm.compress_workspace(16, 60, 4, pamm.PAMM_BF16) == 0         # rows not 16-byte aligned
    assert pamm.compress_workspace(16, 60, 4, pamm.PAMM_F32) > 0           # 60 floats = 240 bytes is fine
    assert pamm.compress_workspace(16, 64, 4, 7) == 0                      # unknown dtype
    assert pamm.grad_workspace(16, 64, 4, 0, pamm.PAMM_F32) == 0
    assert pamm.grad_workspace(16, 64, 4, 12, pamm.PAMM_BF16) == 0         # m rows not 16-byte aligned
    # monotone in b
    assert pamm.compress_workspace(4096, 256, 16, pamm.PAMM_F32) > pamm.compress_workspace(1024, 256, 16, pamm.PAMM_F32)


A = 0x10000   # a 16-byte aligned, non-null fake address: the checks below must fail before it is ever touched
BIG = 1 << 40


def _compress(pamm, X=A, b=64, n=64, k=4, seed=0, dt=1, C=A, f=A, alpha=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_compress(X, b, n, k, ctypes.c_uint64(seed), dt, C, f, alpha, ws, ws_bytes, None)


def _compress_idx(pamm, X=A, b=64, n=64, k=4, idx=A, dt=1, C=A, f=A, alpha=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_compress_idx(X, b, n, k, idx, dt, C, f, alpha, ws, ws_bytes, None)


def _grad(pamm, C=A, f=A, alpha=A, dY=A, b=64, n=64, k=4, m=64, dt=1, dW=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_grad(C, f, alpha, dY, b, n, k, m, dt, dW, ws, ws_bytes, None)


def _contract(pamm, f=A, alpha=A, dY=A, b=64, k=4, m=64, dt=1, Bt=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_contract(f, alpha, dY, b, k, m, dt, Bt, ws, ws_bytes, None)


def test_compress_argument_checks(pamm):
    P = pamm
    for fn in (_compress, _compress_idx):
        assert fn(P, X=None) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, C=None) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, f=None) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, alpha=None) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, X=A + 4) == P.PAMM_ERR_INVALID_ARG          # misaligned
        assert fn(P, k=0) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, k=65) == P.PAMM_ERR_INVALID_ARG             # k > b
        assert fn(P, b=0) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, n=0) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, b=1 << 31, k=4) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, n=60) == P.PAMM_ERR_UNSUPPORTED             # bf16 rows of 120 bytes
        assert fn(P, dt=5) == P.PAMM_ERR_UNSUPPORTED
        assert fn(P, b=1 << 20, k=20000) == P.PAMM_ERR_UNSUPPORTED
        assert fn(P, ws=None) == P.PAMM_ERR_WORKSPACE
        assert fn(P, ws_bytes=16) == P.PAMM_ERR_WORKSPACE
        assert fn(P, ws=A + 8) == P.PAMM_ERR_INVALID_ARG
    assert _compress_idx(P, idx=None) == P.PAMM_ERR_INVALID_ARG


def test_grad_argument_checks(pamm):
    P = pamm
    assert _grad(P, C=None) == P.PAMM_ERR_INVALID_ARG
    assert _grad(P, dW=None) == P.PAMM_ERR_INVALID_ARG
    assert _grad(P, dY=A + 2) == P.PAMM_ERR_INVALID_ARG
    assert _grad(P, m=0) == P.PAMM_ERR_INVALID_ARG
    assert _grad(P, k=65) == P.PAMM_ERR_INVALID_ARG
    assert _grad(P, m=12) == P.PAMM_ERR_UNSUPPORTED
    assert _grad(P, dt=-1) == P.PAMM_ERR_UNSUPPORTED
    assert _grad(P, ws=None) == P.PAMM_ERR_WORKSPACE
    assert _grad(P, ws_bytes=1024) == P.PAMM_ERR_WORKSPACE
    for fn_kw in ("f", "alpha", "dY", "Bt"):
        assert _contract(P, **{fn_kw: None}) == P.PAMM_ERR_INVALID_ARG
    assert _contract(P, m=4, dt=1) == P.PAMM_ERR_UNSUPPORTED
    assert _contract(P, ws_bytes=64) == P.PAMM_ERR_WORKSPACE
    assert _contract(P, k=0) == P.PAMM_ERR_INVALID_ARG


def _compress_eps(pamm, X=A, b=64, n=64, k=4, seed=0, eps=0.5, dt=1, C=A, f=A, alpha=A, eta=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_compress_eps(X, b, n, k, ctypes.c_uint64(seed), ctypes.c_float(eps), dt, C, f, alpha, eta, ws, ws_bytes, None)


def _compress_idx_eps(pamm, X=A, b=64, n=64, k=4, idx=A, eps=0.5, dt=1, C=A, f=A, alpha=A, eta=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_compress_idx_eps(X, b, n, k, idx, ctypes.c_float(eps), dt, C, f, alpha, eta, ws, ws_bytes, None)


def _grad_eps(pamm, C=A, f=A, alpha=A, eta=A, dY=A, b=64, n=64, k=4, m=64, dt=1, dW=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_grad_eps(C, f, alpha, eta, dY, b, n, k, m, dt, dW, ws, ws_bytes, None)


def test_tolerance_argument_checks(pamm):
    """The eps forms refuse a negative or NaN tolerance and a missing or misaligned eta before anything else."""
    P = pamm
    for fn in (_compress_eps, _compress_idx_eps):
        assert fn(P, eps=-0.1) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, eps=float("nan")) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, eta=None) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, eta=A + 2) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, X=None) == P.PAMM_ERR_INVALID_ARG
        assert fn(P, n=60) == P.PAMM_ERR_UNSUPPORTED
        assert fn(P, ws_bytes=16) == P.PAMM_ERR_WORKSPACE
        assert fn(P, eps=float("inf"), ws=None) == P.PAMM_ERR_WORKSPACE        # an infinite tolerance is legal
    assert _compress_idx_eps(P, idx=None) == P.PAMM_ERR_INVALID_ARG
    assert _grad_eps(P, eta=None) == P.PAMM_ERR_INVALID_ARG
    assert _grad_eps(P, eta=A + 1) == P.PAMM_ERR_INVALID_ARG
    assert _grad_eps(P, dW=None) == P.PAMM_ERR_INVALID_ARG
    assert _grad_eps(P, ws_bytes=1024) == P.PAMM_ERR_WORKSPACE


def _grad_out(pamm, C=A, f=A, alpha=A, eta=None, dY=A, b=64, n=64, k=4, m=64, dt=1, out_dt=1, layout=1, dW=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_grad_out(C, f, alpha, eta, dY, b, n, k, m, dt, out_dt, layout, dW, ws, ws_bytes, None)


def test_grad_out_argument_checks(pamm):
    """Element type and orientation of dW are checked on the host like everything else; eta may be absent."""
    P = pamm
    assert _grad_out(P, out_dt=2) == P.PAMM_ERR_UNSUPPORTED
    assert _grad_out(P, layout=2) == P.PAMM_ERR_UNSUPPORTED
    assert _grad_out(P, layout=-1) == P.PAMM_ERR_UNSUPPORTED
    assert _grad_out(P, eta=A + 2) == P.PAMM_ERR_INVALID_ARG
    assert _grad_out(P, dW=None) == P.PAMM_ERR_INVALID_ARG
    assert _grad_out(P, dW=A + 4) == P.PAMM_ERR_INVALID_ARG
    assert _grad_out(P, m=12) == P.PAMM_ERR_UNSUPPORTED
    assert _grad_out(P, k=65) == P.PAMM_ERR_INVALID_ARG
    assert _grad_out(P, ws=None) == P.PAMM_ERR_WORKSPACE
    assert _grad_out(P, eta=A, ws_bytes=1024) == P.PAMM_ERR_WORKSPACE
    # fp32 inputs with rows of 4k+... elements: a bf16 result needs an even row length, which multiples of 4 always are
    assert _grad_out(P, dt=0, n=4, m=4, out_dt=1, layout=0, ws=None) == P.PAMM_ERR_WORKSPACE


def _sketch(pamm, X=A, Pt=A, b=64, n=64, r=8, dt=1, S=A):
    return pamm.lib.pamm_sketch(X, Pt, b, n, r, dt, S, None)


def _sketch_grad(pamm, Pt=A, S=A, dY=A, b=64, n=64, r=8, m=64, dt=1, dW=A, ws=A, ws_bytes=BIG):
    return pamm.lib.pamm_sketch_grad(Pt, S, dY, b, n, r, m, dt, dW, ws, ws_bytes, None)


def test_sketch_argument_checks(pamm):
    P = pamm
    for kw in ("X", "Pt", "S"):
        assert _sketch(P, **{kw: None}) == P.PAMM_ERR_INVALID_ARG
        assert _sketch(P, **{kw: A + 4}) == P.PAMM_ERR_INVALID_ARG
    assert _sketch(P, r=0) == P.PAMM_ERR_INVALID_ARG
    assert _sketch(P, b=4, r=8) == P.PAMM_ERR_INVALID_ARG             # more directions than rows
    assert _sketch(P, r=12) == P.PAMM_ERR_UNSUPPORTED                 # rows of S not 16-byte aligned
    assert _sketch(P, b=256, r=136) == P.PAMM_ERR_UNSUPPORTED         # wider than the widest sketch
    assert _sketch(P, n=60) == P.PAMM_ERR_UNSUPPORTED
    assert _sketch(P, dt=5) == P.PAMM_ERR_UNSUPPORTED
    for kw in ("Pt", "S", "dY", "dW"):
        assert _sketch_grad(P, **{kw: None}) == P.PAMM_ERR_INVALID_ARG
    assert _sketch_grad(P, dt=5) == P.PAMM_ERR_UNSUPPORTED
    assert _sketch_grad(P, m=12) == P.PAMM_ERR_UNSUPPORTED
    assert _sketch_grad(P, m=0) == P.PAMM_ERR_INVALID_ARG
    assert _sketch_grad(P, ws=None) == P.PAMM_ERR_WORKSPACE
    assert _sketch_grad(P, ws_bytes=1024) == P.PAMM_ERR_WORKSPACE
    # the workspace holds one partial row of G per sketch column and chunk, and both operands of the last product
    need = P.sketch_grad_workspace(65536, 2048, 8, 6144, P.PAMM_BF16)
    assert need >= 8 * 6144 * 4 * 2 and need < (64 << 20)
    assert P.sketch_grad_workspace(65536, 2048, 8, 6144, P.PAMM_F32) >= 8 * 6144 * 4 * 2
    assert P.sketch_grad_workspace(65536, 2048, 136, 6144, P.PAMM_BF16) == 0


def test_binding_refuses_cpu_tensors(pamm):
    import torch

    X = torch.zeros(64, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        pamm.compress(X, 4)
