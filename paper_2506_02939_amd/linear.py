"""A linear layer that keeps its input in PAMM's compressed form (Alg. 2: forward pass, Alg. 3: backward pass).

Forward:  Z = X W, then (C, f, alpha) = Compress(flatten(X)); only C, f, alpha (and W) are kept for the backward pass,
          k n + 2 b numbers instead of the b n of X (App. J).
Backward: dW~ = ApproxMM(C, f, alpha, flatten(dZ)),  dX = dZ W^T (exact).

Compress and ApproxMM are the library's calls (pamm.compress / pamm.grad, every step in its HIP kernels).  The two
exact products are ordinary dense GEMMs and go through torch.matmul, i.e. the vendor BLAS; they are not part of the
method.  Nothing here has a CPU path: tensors must live on the GPU.

With `overlap=True` the library's calls run on a second stream (default priority) beside the GEMM that reads the same
matrix: Compress beside Z = X W, ApproxMM beside dX = dZ W^T, joined again before the pass returns.  The GEMM is bound
by the matrix cores and leaves HBM idle; the call beside it finds part of X / dZ in the caches and most of its time
disappears behind the GEMM (Alg. 2-3 leave the order of the two steps of each pass open).  Results are the same bit
for bit.
"""
from __future__ import annotations

import math

import torch

from . import pamm


_side_streams: dict = {}


def _side_stream(device) -> torch.cuda.Stream:
    key = torch.device(device).index if torch.device(device).index is not None else torch.cuda.current_device()
    if key not in _side_streams:
        _side_streams[key] = torch.cuda.Stream(device=key)          # default priority
    return _side_streams[key]


def generators_for(b: int, r: float) -> int:
    """k = ceil(r b), at least 1 and at most b (Sec. 4.1)."""
    return max(1, min(b, math.ceil(r * b)))


class _PammLinear(torch.autograd.Function):
    @staticmethod
    def forward(ctx, X, W, k, seed, eps, out_by_in, overlap):
        n = X.shape[-1]
        x2 = X.reshape(-1, n)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        x2 = x2.detach()
        if overlap:
            # outputs are allocated on the caller's stream; only the kernels move to the second one
            b = x2.shape[0]
            comp = pamm.Compressed(torch.empty(k, n, dtype=x2.dtype, device=x2.device),
                                   torch.empty(b, dtype=torch.int32, device=x2.device),
                                   torch.empty(b, dtype=torch.float32, device=x2.device),
                                   torch.empty(1, dtype=torch.int32, device=x2.device) if eps is not None else None)
            cur, side = torch.cuda.current_stream(), _side_stream(x2.device)
            side.wait_stream(cur)
            with torch.cuda.stream(side):
                pamm.compress(x2, k, seed=seed, eps=eps, out=comp)
            Z = torch.matmul(X, W.t() if out_by_in else W)
            cur.wait_stream(side)
        else:
            Z = torch.matmul(X, W.t() if out_by_in else W)
            comp = pamm.compress(x2, k, seed=seed, eps=eps)
        saved = [comp.C, comp.f, comp.alpha, W] + ([comp.eta] if comp.eta is not None else [])
        ctx.save_for_backward(*saved)
        ctx.out_by_in = out_by_in
        ctx.overlap = overlap
        ctx.x_shape = X.shape
        return Z

    @staticmethod
    def backward(ctx, dZ):
        C, f, alpha, W = ctx.saved_tensors[:4]
        eta = ctx.saved_tensors[4] if len(ctx.saved_tensors) > 4 else None
        dX = dW = None
        side = None
        if ctx.needs_input_grad[1]:
            dz2 = dZ.reshape(-1, dZ.shape[-1])
            if not dz2.is_contiguous():
                dz2 = dz2.contiguous()
            if dz2.dtype != C.dtype:
                dz2 = dz2.to(C.dtype)
            if ctx.overlap and ctx.needs_input_grad[0]:
                k, n = C.shape
                m = dz2.shape[1]
                dW = torch.empty((m, n) if ctx.out_by_in else (n, m), dtype=W.dtype, device=W.device)
                cur, side = torch.cuda.current_stream(), _side_stream(W.device)
                side.wait_stream(cur)
                with torch.cuda.stream(side):
                    pamm.grad(C, f, alpha, dz2, eta=eta, out_dtype=W.dtype, transposed=ctx.out_by_in, out=dW)
            else:
                dW = pamm.grad(C, f, alpha, dz2, eta=eta, out_dtype=W.dtype, transposed=ctx.out_by_in)
        if ctx.needs_input_grad[0]:
            dX = torch.matmul(dZ, W if ctx.out_by_in else W.t()).reshape(ctx.x_shape)
        if side is not None:
            torch.cuda.current_stream().wait_stream(side)
        return dX, dW, None, None, None, None, None


def pamm_linear(X: torch.Tensor, W: torch.Tensor, *, r: float | None = 1.0 / 512, k: int | None = None, seed: int = 0,
                eps: float | None = None, out_by_in: bool = False, overlap: bool = False) -> torch.Tensor:
    """Z = X W for X of shape (..., n) and W of shape n x m (the paper's orientation), or, with `out_by_in`, W of
    shape m x n and Z = X W^T (the orientation of torch.nn.Linear.weight).  In the backward pass the gradient of W is
    PAMM's estimate from k = ceil(r b) generators (or `k` as given) sampled with `seed`; `eps` switches the
    neighbourhood condition of Eq. 2 and the factor beta on.  The gradient of X is exact.  A training loop passes a
    fresh seed every step (Alg. 1 samples anew on every call).  `overlap`: run Compress / ApproxMM on a second stream
    beside the exact GEMM of the same pass (see the module's head)."""
    b = X.numel() // X.shape[-1]
    kk = generators_for(b, r) if k is None else k
    return _PammLinear.apply(X, W, kk, seed, eps, out_by_in, overlap)
