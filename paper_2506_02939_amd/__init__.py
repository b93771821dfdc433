"""MI355X-native PAMM hot path: Compress (X -> C, f, alpha) and ApproxMM (C, f, alpha, dY -> dW~).

``paper_2506_02939_amd.pamm`` is the thin binding over the C-ABI library (HIP kernels for gfx950);
``paper_2506_02939_amd.linear`` is the linear layer of Alg. 2-3 on top of it;
``paper_2506_02939_amd.workloads`` draws the seeded synthetic inputs.  Nothing is imported eagerly,
so the input generator can be used without the compiled library.
"""
__all__ = ["pamm", "workloads", "linear"]
