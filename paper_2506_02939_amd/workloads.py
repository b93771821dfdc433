"""Seeded synthetic inputs: token-redundant activations X (b x n) and upstream gradients dY (b x m).

This module is shared by the GPU tests, the benchmark and the CPU oracle's tests.
It holds no arithmetic of the method itself: it only draws inputs.  It stands in
for the recorded LLaMA activations the paper measures on (Sec. 4; App. H), which
are not available: rows cluster around a limited set of directions with varying
scale, may repeat exactly (padding) or resemble their neighbours in the sequence,
which are the three sources of token redundancy the paper's introduction names.

Recipe (all draws from one ``torch.Generator`` on the CPU, seeded per workload):
  centres   mu_c ~ N(0, I_n)
  label     z_i uniform over centres,   scale s_i ~ U(0.5, 2)
  iid       X_i = s_i * mu_{z_i} + sigma * N(0, I_n)
  ar1       per sequence h_0 = mu_{z_0}, h_t = rho*h_{t-1} + sqrt(1-rho^2)*mu_{z_t};  X_t = s_t*h_t + sigma*N(0, I_n)
  padding   one vector p (drawn like a row) per batch; the last ceil(pad_frac*L) positions of
            every sequence are bit-identical copies of p
  dY        N(0, 0.1^2)  (variance 1e-2)
  Pt        for the random-projection baseline (Sec. 4.6): r directions, entries N(0, 1/r), so that E[P P^T] = I
Values are drawn in float32 and then rounded once to the workload's element type;
the rounded values are what every consumer sees.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    seqs: int          # sequences in the batch
    seq_len: int       # tokens per sequence;  b = seqs * seq_len
    n: int             # hidden size (columns of X)
    m: int             # fused Q|K|V width (columns of dY)
    k: int             # generators
    dtype: str         # "f32" or "bf16"
    centres: int
    sigma: float
    structure: str = "iid"     # "iid" or "ar1"
    rho: float = 0.0
    pad_frac: float = 0.0
    seed: int = 0              # seed of the input generator (not of the sampler)

    @property
    def b(self) -> int:
        return self.seqs * self.seq_len

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny", 8, 256, 256, 768, 16, "f32", 64, 0.1, seed=0),
        Workload("llama60m", 32, 256, 512, 1536, 16, "bf16", 256, 0.1, pad_frac=0.10, seed=1),
        Workload("llama350m", 64, 512, 1024, 3072, 64, "bf16", 1024, 0.1, structure="ar1", rho=0.9, seed=2),
        Workload("llama1b", 64, 1024, 2048, 6144, 128, "bf16", 4096, 0.2, seed=3),
        Workload("llama7b_k32", 4, 4096, 4096, 12288, 32, "bf16", 2048, 0.2, pad_frac=0.20, seed=4),
        Workload("llama7b_k256", 4, 4096, 4096, 12288, 256, "bf16", 2048, 0.2, pad_frac=0.20, seed=4),
        Workload("llama7b_k1024", 4, 4096, 4096, 12288, 1024, "bf16", 2048, 0.2, pad_frac=0.20, seed=4),
    ]
}


def scaled(w: Workload, *, seqs=None, seq_len=None, n=None, m=None, k=None, centres=None, name=None) -> Workload:
    """The same recipe at another size (for tests that need the oracle to finish quickly)."""
    kw = {}
    for key, val in (("seqs", seqs), ("seq_len", seq_len), ("n", n), ("m", m), ("k", k), ("centres", centres), ("name", name)):
        if val is not None:
            kw[key] = val
    return replace(w, **kw)


def generate_x(w: Workload) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed)
    b, n = w.b, w.n
    mu = torch.randn(w.centres, n, generator=g)
    z = torch.randint(0, w.centres, (b,), generator=g)
    s = torch.rand(b, generator=g) * 1.5 + 0.5
    if w.structure == "iid":
        x = mu[z]
    elif w.structure == "ar1":
        mz = mu[z].view(w.seqs, w.seq_len, n)
        h = torch.empty_like(mz)
        h[:, 0] = mz[:, 0]
        c = math.sqrt(1.0 - w.rho * w.rho)
        for t in range(1, w.seq_len):
            h[:, t] = w.rho * h[:, t - 1] + c * mz[:, t]
        x = h.view(b, n)
    else:
        raise ValueError(w.structure)
    x = x * s[:, None]
    # noise in slabs so the peak footprint stays near 2x the matrix
    step = max(1, (1 << 26) // n)
    for r0 in range(0, b, step):
        r1 = min(b, r0 + step)
        x[r0:r1] += w.sigma * torch.randn(r1 - r0, n, generator=g)
    if w.pad_frac > 0.0:
        pz = int(torch.randint(0, w.centres, (1,), generator=g))
        ps = float(torch.rand(1, generator=g)) * 1.5 + 0.5
        p = ps * mu[pz] + w.sigma * torch.randn(n, generator=g)
        npad = math.ceil(w.pad_frac * w.seq_len)
        x.view(w.seqs, w.seq_len, n)[:, w.seq_len - npad:, :] = p
    return x.to(w.torch_dtype).contiguous()


def generate_dy(w: Workload) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed + 7919)
    b, m = w.b, w.m
    out = torch.empty(b, m, dtype=w.torch_dtype)
    step = max(1, (1 << 26) // m)
    for r0 in range(0, b, step):
        r1 = min(b, r0 + step)
        out[r0:r1] = (0.1 * torch.randn(r1 - r0, m, generator=g)).to(w.torch_dtype)
    return out


def generate(w: Workload):
    """(X, dY) as contiguous CPU tensors of the workload's element type."""
    return generate_x(w), generate_dy(w)


def sketch_directions(w: Workload, r: int) -> torch.Tensor:
    """Pt (r x n): the transpose of the random projection P of the sketch baseline, entries N(0, 1/r)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed + 104729)
    return (torch.randn(r, w.n, generator=g) / math.sqrt(r)).to(w.torch_dtype).contiguous()


def matched_sketch_width(w: Workload) -> int:
    """Sketch width whose b r stored numbers are at least the k n + 2 b that PAMM keeps, as a whole 16-byte row."""
    r = -(-(w.k * w.n + 2 * w.b) // w.b)
    return max(8, -(-r // 8) * 8)
