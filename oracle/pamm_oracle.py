"""ctypes front end of the fp64 CPU oracle in ``pamm_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  The arithmetic is
all in the C file (which cites the passages of the paper it follows); this
module only compiles it with gcc, marshals numpy arrays and returns numpy
arrays.  It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pamm_oracle.c")
_LIB = os.path.join(_HERE, "libpamm_oracle.so")

F32, BF16, F64 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32p, f64p, vp = ctypes.c_int64, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double), ctypes.c_void_p
        lib.pamm_oracle_threads.restype = ctypes.c_int
        lib.pamm_oracle_set_threads.argtypes = [ctypes.c_int]
        lib.pamm_oracle_splitmix64.argtypes = [ctypes.c_uint64, i64, ctypes.POINTER(ctypes.c_uint64)]
        lib.pamm_oracle_sample.argtypes = [i64, i64, ctypes.c_uint64, i32p]
        lib.pamm_oracle_sample.restype = ctypes.c_int
        lib.pamm_oracle_compress.argtypes = [vp, ctypes.c_int, i64, i64, i64, i32p, ctypes.c_double, f64p, i32p, f64p, f64p, f64p,
                                             i32p, f64p, f64p, ctypes.POINTER(ctypes.c_int64)]
        lib.pamm_oracle_compress.restype = ctypes.c_int
        lib.pamm_oracle_beta.argtypes = [i64, i64]
        lib.pamm_oracle_beta.restype = ctypes.c_double
        lib.pamm_oracle_grad.argtypes = [f64p, i32p, f64p, vp, ctypes.c_int, i64, i64, i64, i64, ctypes.c_double, f64p, f64p]
        lib.pamm_oracle_grad.restype = ctypes.c_int
        lib.pamm_oracle_bounded.argtypes = [ctypes.c_uint64, ctypes.c_uint64, i64, ctypes.POINTER(ctypes.c_uint64)]
        lib.pamm_oracle_bounded.restype = ctypes.c_int
        lib.pamm_oracle_sketch.argtypes = [vp, ctypes.c_int, vp, ctypes.c_int, i64, i64, i64, f64p]
        lib.pamm_oracle_sketch.restype = ctypes.c_int
        lib.pamm_oracle_sketch_grad.argtypes = [vp, ctypes.c_int, vp, ctypes.c_int, vp, ctypes.c_int, i64, i64, i64, i64, f64p, f64p]
        lib.pamm_oracle_sketch_grad.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().pamm_oracle_threads())


def set_threads(t: int) -> None:
    _load().pamm_oracle_set_threads(int(t))


def as_raw(x):
    """(contiguous numpy array, element-type code) for a matrix given as a numpy array
    (float32, float64, or uint16 holding bfloat16 bit patterns) or as a CPU torch tensor
    (float32, float64 or bfloat16).  No value is changed."""
    if not isinstance(x, np.ndarray):
        import torch  # only needed to re-view bfloat16 storage

        t = x.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            x = t.view(torch.int16).numpy().view(np.uint16)
        else:
            x = t.numpy()
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        return x, F32
    if x.dtype == np.uint16:
        return x, BF16
    if x.dtype == np.float64:
        return x, F64
    raise TypeError(f"unsupported element type {x.dtype}")


def to_f64(x) -> np.ndarray:
    """Exact widening of a float32 / bfloat16-bits / float64 matrix to float64 (for the tests' own numpy checks)."""
    a, code = as_raw(x)
    if code == BF16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _p(a, ty):
    return a.ctypes.data_as(ctypes.POINTER(ty))


def splitmix64(seed: int, count: int) -> np.ndarray:
    out = np.empty(count, dtype=np.uint64)
    _load().pamm_oracle_splitmix64(ctypes.c_uint64(seed), count, _p(out, ctypes.c_uint64))
    return out


def bounded(seed: int, u: int, count: int) -> np.ndarray:
    """`count` consecutive draws of the sampler's bounded(u) (uniform on [0,u) by rejection) from one seeded generator."""
    out = np.empty(count, dtype=np.uint64)
    rc = _load().pamm_oracle_bounded(ctypes.c_uint64(seed & (2**64 - 1)), ctypes.c_uint64(u), count, _p(out, ctypes.c_uint64))
    if rc != 0:
        raise ValueError("pamm_oracle_bounded: bad arguments")
    return out


def sample(b: int, k: int, seed: int) -> np.ndarray:
    idx = np.empty(k, dtype=np.int32)
    rc = _load().pamm_oracle_sample(b, k, ctypes.c_uint64(seed & (2**64 - 1)), _p(idx, ctypes.c_int32))
    if rc != 0:
        raise ValueError("pamm_oracle_sample: bad arguments")
    return idx


@dataclass
class Compressed:
    idx: np.ndarray      # k int32, generator rows in draw order
    C: np.ndarray        # k x n float64
    f: np.ndarray        # b int32
    alpha: np.ndarray    # b float64
    best: np.ndarray     # b float64, score of the chosen generator
    second: np.ndarray   # b float64, best score among the other generators (-1 if k == 1)
    jsecond: np.ndarray  # b int32, generator attaining `second` (-1 if k == 1)
    resid: np.ndarray    # b float64, ||A_i - alpha_i C_f(i)||_2 before the neighbourhood mask
    rownorm: np.ndarray  # b float64, ||A_i||_2
    eta: int             # rows dropped by the neighbourhood condition
    beta: float          # b / (b - eta)


def compress(X, k: int, seed: int = 0, idx=None, eps: float = float("inf")) -> Compressed:
    """Compress(A, k, eps).  `idx` overrides the sampler (caller-chosen generators); eps = inf drops no row."""
    a, code = as_raw(X)
    b, n = a.shape
    idx = sample(b, k, seed) if idx is None else np.ascontiguousarray(idx, dtype=np.int32)
    assert idx.shape == (k,)
    C = np.empty((k, n), dtype=np.float64)
    f = np.empty(b, dtype=np.int32)
    alpha = np.empty(b, dtype=np.float64)
    best = np.empty(b, dtype=np.float64)
    second = np.empty(b, dtype=np.float64)
    jsecond = np.empty(b, dtype=np.int32)
    resid = np.empty(b, dtype=np.float64)
    rownorm = np.empty(b, dtype=np.float64)
    eta = ctypes.c_int64(0)
    eps_c = -1.0 if (eps is None or np.isinf(eps)) else float(eps)
    if eps_c < 0.0 and not (eps is None or np.isinf(eps)):
        raise ValueError("eps must be >= 0")
    rc = _load().pamm_oracle_compress(
        a.ctypes.data_as(ctypes.c_void_p), code, b, n, k, _p(idx, ctypes.c_int32), eps_c,
        _p(C, ctypes.c_double), _p(f, ctypes.c_int32), _p(alpha, ctypes.c_double),
        _p(best, ctypes.c_double), _p(second, ctypes.c_double), _p(jsecond, ctypes.c_int32),
        _p(resid, ctypes.c_double), _p(rownorm, ctypes.c_double), ctypes.byref(eta))
    if rc != 0:
        raise ValueError("pamm_oracle_compress: bad arguments")
    beta = float(_load().pamm_oracle_beta(b, eta.value))
    return Compressed(idx, C, f, alpha, best, second, jsecond, resid, rownorm, int(eta.value), beta)


def grad(C, f, alpha, dY, beta: float = 1.0):
    """ApproxMM(C, alpha, f, B): returns (Btilde k x m, Otilde = beta C^T Btilde, n x m), both float64."""
    C = np.ascontiguousarray(C, dtype=np.float64)
    f = np.ascontiguousarray(f, dtype=np.int32)
    alpha = np.ascontiguousarray(alpha, dtype=np.float64)
    y, code = as_raw(dY)
    k, n = C.shape
    b, m = y.shape
    assert f.shape == (b,) and alpha.shape == (b,)
    Bt = np.empty((k, m), dtype=np.float64)
    O = np.empty((n, m), dtype=np.float64)
    rc = _load().pamm_oracle_grad(
        _p(C, ctypes.c_double), _p(f, ctypes.c_int32), _p(alpha, ctypes.c_double),
        y.ctypes.data_as(ctypes.c_void_p), code, b, n, k, m, float(beta), _p(Bt, ctypes.c_double), _p(O, ctypes.c_double))
    if rc != 0:
        raise ValueError("pamm_oracle_grad: bad arguments")
    return Bt, O


def sketch(X, Pt) -> np.ndarray:
    """S = X P for P given through its transpose Pt (r x n): S[i][j] = <X_i, Pt_j>, b x r float64, not rounded
    (the random-projection baseline of Sec. 4.6)."""
    x, xcode = as_raw(X)
    p, pcode = as_raw(Pt)
    b, n = x.shape
    r, n2 = p.shape
    assert n2 == n
    S = np.empty((b, r), dtype=np.float64)
    rc = _load().pamm_oracle_sketch(x.ctypes.data_as(ctypes.c_void_p), xcode, p.ctypes.data_as(ctypes.c_void_p), pcode,
                                    b, n, r, _p(S, ctypes.c_double))
    if rc != 0:
        raise ValueError("pamm_oracle_sketch: bad arguments")
    return S


def sketch_grad(Pt, S, dY):
    """The sketch's estimate of X^T dY: returns (G = S^T dY, r x m; O = P G = Pt^T G, n x m), both float64.  S is the
    stored sketch in its own element type (numpy float32 / float64 / bfloat16 bits, or a CPU torch tensor)."""
    p, pcode = as_raw(Pt)
    s, scode = as_raw(S)
    y, ycode = as_raw(dY)
    r, n = p.shape
    b, m = y.shape
    assert s.shape == (b, r)
    G = np.empty((r, m), dtype=np.float64)
    O = np.empty((n, m), dtype=np.float64)
    rc = _load().pamm_oracle_sketch_grad(p.ctypes.data_as(ctypes.c_void_p), pcode, s.ctypes.data_as(ctypes.c_void_p), scode,
                                         y.ctypes.data_as(ctypes.c_void_p), ycode, b, n, r, m,
                                         _p(G, ctypes.c_double), _p(O, ctypes.c_double))
    if rc != 0:
        raise ValueError("pamm_oracle_sketch_grad: bad arguments")
    return G, O
