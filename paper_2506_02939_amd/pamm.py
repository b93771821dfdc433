"""Thin binding over libpamm's C ABI (include/pamm.h): argument marshalling only.

Every step of Compress / ApproxMM runs in the HIP kernels of ``libpamm.so``; torch is used here
for device memory and the current stream.  There is no fallback: if the library is missing, or no
MI355X is present when a compute call is made, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpamm.so")

PAMM_OK = 0
PAMM_ERR_INVALID_ARG, PAMM_ERR_UNSUPPORTED, PAMM_ERR_WORKSPACE, PAMM_ERR_DEVICE = 1, 2, 3, 4
PAMM_F32, PAMM_BF16 = 0, 1
PAMM_DW_N_BY_M, PAMM_DW_M_BY_N = 0, 1

EXPORTS = [
    "pamm_status_string", "pamm_compress_workspace", "pamm_grad_workspace", "pamm_sample_indices",
    "pamm_compress", "pamm_compress_idx", "pamm_compress_eps", "pamm_compress_idx_eps", "pamm_grad", "pamm_grad_eps",
    "pamm_grad_out", "pamm_grad_static", "pamm_contract",
    "pamm_sketch_grad_workspace", "pamm_sketch", "pamm_sketch_grad",
    "pamm_profile_begin", "pamm_profile_end", "pamm_kernel_name",
    "pamm_debug_set_plan", "pamm_debug_bounded",
]
NUM_KERNELS = 10


class PammError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2506_02939_amd.build` "
            "(hipcc, gfx950). There is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    i64, u64, vp, sz, ci = ctypes.c_int64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.pamm_status_string.argtypes = [ci]
    lib.pamm_status_string.restype = ctypes.c_char_p
    lib.pamm_compress_workspace.argtypes = [i64, i64, i64, ci]
    lib.pamm_compress_workspace.restype = sz
    lib.pamm_grad_workspace.argtypes = [i64, i64, i64, i64, ci]
    lib.pamm_grad_workspace.restype = sz
    lib.pamm_sample_indices.argtypes = [i64, i64, u64, vp]
    lib.pamm_sample_indices.restype = ci
    lib.pamm_compress.argtypes = [vp, i64, i64, i64, u64, ci, vp, vp, vp, vp, sz, vp]
    lib.pamm_compress.restype = ci
    lib.pamm_compress_idx.argtypes = [vp, i64, i64, i64, vp, ci, vp, vp, vp, vp, sz, vp]
    lib.pamm_compress_idx.restype = ci
    lib.pamm_compress_eps.argtypes = [vp, i64, i64, i64, u64, ctypes.c_float, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.pamm_compress_eps.restype = ci
    lib.pamm_compress_idx_eps.argtypes = [vp, i64, i64, i64, vp, ctypes.c_float, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.pamm_compress_idx_eps.restype = ci
    lib.pamm_grad.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.pamm_grad.restype = ci
    lib.pamm_grad_eps.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.pamm_grad_eps.restype = ci
    lib.pamm_grad_out.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, ci, vp, vp, sz, vp]
    lib.pamm_grad_out.restype = ci
    lib.pamm_grad_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, ci, vp, vp]
    lib.pamm_grad_static.restype = ci
    lib.pamm_contract.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.pamm_contract.restype = ci
    lib.pamm_sketch_grad_workspace.argtypes = [i64, i64, i64, i64, ci]
    lib.pamm_sketch_grad_workspace.restype = sz
    lib.pamm_sketch.argtypes = [vp, vp, i64, i64, i64, ci, vp, vp]
    lib.pamm_sketch.restype = ci
    lib.pamm_sketch_grad.argtypes = [vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.pamm_sketch_grad.restype = ci
    lib.pamm_profile_begin.argtypes = []
    lib.pamm_profile_begin.restype = ci
    lib.pamm_profile_end.argtypes = [vp, vp]
    lib.pamm_profile_end.restype = ci
    lib.pamm_kernel_name.argtypes = [ci]
    lib.pamm_kernel_name.restype = ctypes.c_char_p
    lib.pamm_debug_set_plan.argtypes = [vp]
    lib.pamm_debug_set_plan.restype = ci
    lib.pamm_debug_bounded.argtypes = [u64, u64, i64, vp]
    lib.pamm_debug_bounded.restype = ci
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.pamm_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != PAMM_OK:
        raise PammError(status, what)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PAMM_F32
    if t.dtype == torch.bfloat16:
        return PAMM_BF16
    raise PammError(PAMM_ERR_UNSUPPORTED, f"element type {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU (no CPU path exists)")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def compress_workspace(b: int, n: int, k: int, dtype: int) -> int:
    return int(lib.pamm_compress_workspace(b, n, k, dtype))


def grad_workspace(b: int, n: int, k: int, m: int, dtype: int) -> int:
    return int(lib.pamm_grad_workspace(b, n, k, m, dtype))


def sample_indices(b: int, k: int, seed: int) -> torch.Tensor:
    """pamm_sample_indices: k generator rows for (b, seed), a CPU int32 tensor in draw order."""
    idx = torch.empty(max(k, 0), dtype=torch.int32)
    _check(lib.pamm_sample_indices(b, k, ctypes.c_uint64(seed & (2**64 - 1)), idx.data_ptr()), "pamm_sample_indices")
    return idx


def _workspace(nbytes: int, device, ws):
    if ws is None:
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    return ws


@dataclass
class Compressed:
    C: torch.Tensor       # k x n, element type of X
    f: torch.Tensor       # b int32
    alpha: torch.Tensor   # b fp32
    eta: torch.Tensor | None = None     # one int32 on the device: rows dropped by the neighbourhood condition (eps given)


def compress(X: torch.Tensor, k: int, seed: int = 0, *, idx: torch.Tensor | None = None, eps: float | None = None,
             out: Compressed | None = None, ws: torch.Tensor | None = None) -> Compressed:
    """pamm_compress (or pamm_compress_idx when `idx`, a device int32 tensor of k rows, is given); with `eps` the
    _eps forms, which also fill `eta`."""
    b, n = X.shape
    dt = _dtype_code(X)
    xp = _dev(X, "X")
    if out is None:
        out = Compressed(torch.empty(k, n, dtype=X.dtype, device=X.device),
                         torch.empty(b, dtype=torch.int32, device=X.device),
                         torch.empty(b, dtype=torch.float32, device=X.device))
    nbytes = compress_workspace(b, n, k, dt)
    if nbytes == 0:
        # let the library name the problem
        ws = _workspace(16, X.device, ws)
    else:
        ws = _workspace(nbytes, X.device, ws)
    if eps is not None:
        if out.eta is None:
            out.eta = torch.empty(1, dtype=torch.int32, device=X.device)
        if idx is None:
            st = lib.pamm_compress_eps(xp, b, n, k, ctypes.c_uint64(seed & (2**64 - 1)), ctypes.c_float(eps), dt, out.C.data_ptr(),
                                       out.f.data_ptr(), out.alpha.data_ptr(), out.eta.data_ptr(), ws.data_ptr(), ws.numel(),
                                       _stream())
            _check(st, "pamm_compress_eps")
        else:
            st = lib.pamm_compress_idx_eps(xp, b, n, k, _dev(idx, "idx"), ctypes.c_float(eps), dt, out.C.data_ptr(),
                                           out.f.data_ptr(), out.alpha.data_ptr(), out.eta.data_ptr(), ws.data_ptr(), ws.numel(),
                                           _stream())
            _check(st, "pamm_compress_idx_eps")
    elif idx is None:
        st = lib.pamm_compress(xp, b, n, k, ctypes.c_uint64(seed & (2**64 - 1)), dt, out.C.data_ptr(), out.f.data_ptr(),
                               out.alpha.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
        _check(st, "pamm_compress")
    else:
        st = lib.pamm_compress_idx(xp, b, n, k, _dev(idx, "idx"), dt, out.C.data_ptr(), out.f.data_ptr(),
                                   out.alpha.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
        _check(st, "pamm_compress_idx")
    return out


def grad(C: torch.Tensor, f: torch.Tensor, alpha: torch.Tensor, dY: torch.Tensor, *, eta: torch.Tensor | None = None,
         out_dtype: torch.dtype | None = None, transposed: bool = False, out: torch.Tensor | None = None,
         ws: torch.Tensor | None = None) -> torch.Tensor:
    """pamm_grad: dW (n x m, fp32) = C^T Btilde; with `eta` (device int32) pamm_grad_eps: beta C^T Btilde.
    With `out_dtype` (torch.float32 or torch.bfloat16) or `transposed` (dW as m x n) given: pamm_grad_out."""
    k, n = C.shape
    b, m = dY.shape
    dt = _dtype_code(dY)
    if C.dtype != dY.dtype:
        raise PammError(PAMM_ERR_UNSUPPORTED, "C and dY differ in element type")
    plain = out_dtype is None and not transposed
    odt = torch.float32 if out_dtype is None else out_dtype
    shape = (m, n) if transposed else (n, m)
    if out is None:
        out = torch.empty(*shape, dtype=odt, device=dY.device)
    elif out.dtype != odt or tuple(out.shape) != shape:
        raise ValueError(f"out must be {shape} of {odt}")
    ws = _workspace(grad_workspace(b, n, k, m, dt), dY.device, ws)
    if not plain:
        st = lib.pamm_grad_out(_dev(C, "C"), _dev(f, "f"), _dev(alpha, "alpha"), None if eta is None else _dev(eta, "eta"),
                               _dev(dY, "dY"), b, n, k, m, dt, _dtype_code(out), PAMM_DW_M_BY_N if transposed else PAMM_DW_N_BY_M,
                               _dev(out, "out"), ws.data_ptr(), ws.numel(), _stream())
        _check(st, "pamm_grad_out")
    elif eta is None:
        st = lib.pamm_grad(_dev(C, "C"), _dev(f, "f"), _dev(alpha, "alpha"), _dev(dY, "dY"), b, n, k, m, dt, _dev(out, "out"),
                           ws.data_ptr(), ws.numel(), _stream())
        _check(st, "pamm_grad")
    else:
        st = lib.pamm_grad_eps(_dev(C, "C"), _dev(f, "f"), _dev(alpha, "alpha"), _dev(eta, "eta"), _dev(dY, "dY"), b, n, k, m, dt,
                               _dev(out, "out"), ws.data_ptr(), ws.numel(), _stream())
        _check(st, "pamm_grad_eps")
    return out


STATIC_SCRATCH_BYTES = 16 << 20


def grad_static(C: torch.Tensor, f: torch.Tensor, alpha: torch.Tensor, dY: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """pamm_grad_static: pamm_grad with the library's own static scratch array; the caller passes inputs and `out`
    (n x m fp32) only, and nothing is allocated on either side."""
    k, n = C.shape
    b, m = dY.shape
    st = lib.pamm_grad_static(_dev(C, "C"), _dev(f, "f"), _dev(alpha, "alpha"), _dev(dY, "dY"), b, n, k, m, _dtype_code(dY),
                              _dev(out, "out"), _stream())
    _check(st, "pamm_grad_static")
    return out


def sketch_grad_workspace(b: int, n: int, r: int, m: int, dtype: int) -> int:
    return int(lib.pamm_sketch_grad_workspace(b, n, r, m, dtype))


def sketch(X: torch.Tensor, Pt: torch.Tensor, *, out: torch.Tensor | None = None) -> torch.Tensor:
    """pamm_sketch: S (b x r, element type of X) = X Pt^T, the sketch the random-projection baseline keeps."""
    b, n = X.shape
    r, n2 = Pt.shape
    if n2 != n or Pt.dtype != X.dtype:
        raise PammError(PAMM_ERR_INVALID_ARG, "Pt must be r x n of X's element type")
    if out is None:
        out = torch.empty(b, r, dtype=X.dtype, device=X.device)
    st = lib.pamm_sketch(_dev(X, "X"), _dev(Pt, "Pt"), b, n, r, _dtype_code(X), _dev(out, "out"), _stream())
    _check(st, "pamm_sketch")
    return out


def sketch_grad(Pt: torch.Tensor, S: torch.Tensor, dY: torch.Tensor, *, out: torch.Tensor | None = None,
                ws: torch.Tensor | None = None) -> torch.Tensor:
    """pamm_sketch_grad: dW (n x m, fp32) = Pt^T (S^T dY), the baseline's estimate of X^T dY."""
    r, n = Pt.shape
    b, m = dY.shape
    if tuple(S.shape) != (b, r) or S.dtype != dY.dtype or Pt.dtype != dY.dtype:
        raise PammError(PAMM_ERR_INVALID_ARG, "S must be b x r, and Pt, S, dY of one element type")
    dt = _dtype_code(dY)
    if out is None:
        out = torch.empty(n, m, dtype=torch.float32, device=dY.device)
    ws = _workspace(sketch_grad_workspace(b, n, r, m, dt), dY.device, ws)
    st = lib.pamm_sketch_grad(_dev(Pt, "Pt"), _dev(S, "S"), _dev(dY, "dY"), b, n, r, m, dt, _dev(out, "out"), ws.data_ptr(),
                              ws.numel(), _stream())
    _check(st, "pamm_sketch_grad")
    return out


def contract(f: torch.Tensor, alpha: torch.Tensor, dY: torch.Tensor, k: int, *, ws: torch.Tensor | None = None) -> torch.Tensor:
    """pamm_contract: Btilde (k x m, fp32), the contraction stage of ApproxMM alone."""
    b, m = dY.shape
    dt = _dtype_code(dY)
    out = torch.empty(k, m, dtype=torch.float32, device=dY.device)
    n_any = 8
    ws = _workspace(grad_workspace(b, n_any, k, m, dt), dY.device, ws)
    st = lib.pamm_contract(_dev(f, "f"), _dev(alpha, "alpha"), _dev(dY, "dY"), b, k, m, dt, out.data_ptr(), ws.data_ptr(),
                           ws.numel(), _stream())
    _check(st, "pamm_contract")
    return out


class _DebugPlan(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int) for name in ("score_tg", "score_nw", "piece_rows", "contract_w", "sort_one_rows", "small_tiles")]


def debug_set_plan(**overrides: int) -> None:
    """pamm_debug_set_plan (test hook): force launch-plan fields; no arguments clears every override."""
    if not overrides:
        _check(lib.pamm_debug_set_plan(None), "pamm_debug_set_plan")
        return
    plan = _DebugPlan(**{k: int(v) for k, v in overrides.items()})
    _check(lib.pamm_debug_set_plan(ctypes.addressof(plan)), "pamm_debug_set_plan")


def debug_bounded(seed: int, range_: int, count: int) -> list:
    """pamm_debug_bounded (test hook): `count` draws of the sampler's bounded step on [0, range_)."""
    out = (ctypes.c_uint64 * max(count, 1))()
    _check(lib.pamm_debug_bounded(ctypes.c_uint64(seed & (2**64 - 1)), ctypes.c_uint64(range_), count, ctypes.addressof(out)),
           "pamm_debug_bounded")
    return [int(out[i]) for i in range(count)]


def profile_begin() -> None:
    _check(lib.pamm_profile_begin(), "pamm_profile_begin")


def profile_end() -> dict:
    """{kernel name: (total milliseconds, launches)} for the kernels launched since profile_begin()."""
    ms = (ctypes.c_double * NUM_KERNELS)()
    n = (ctypes.c_int64 * NUM_KERNELS)()
    _check(lib.pamm_profile_end(ctypes.addressof(ms), ctypes.addressof(n)), "pamm_profile_end")
    return {lib.pamm_kernel_name(i).decode(): (float(ms[i]), int(n[i])) for i in range(NUM_KERNELS) if n[i] > 0}
