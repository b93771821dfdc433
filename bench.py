#!/usr/bin/env python3
"""Benchmark of the PAMM hot path on one MI355X: one step = pamm_compress + pamm_grad over one synthetic batch.

Prints ONE JSON line.  `value` is tokens/s = b / (t_compress + t_grad) on the headline workload (the 1B-shaped layer)
with X and dY resident in HBM before the timed region; consecutive steps rotate through `--sets` copies of the inputs
so that a step finds none of its inputs in the Infinity Cache.  `roofline` covers the dominant kernel (k_contract, the
single pass over dY): algorithmic bytes per launch divided by its mean duration, the latter measured here with HIP
events on the launch stream (the library's own per-kernel event hooks) over a second run of the same K steps;
`roofline_kernels` gives the same figures for all three hot kernels (score, contraction, small product), against the
HBM peak and, where the kernel is a matrix product that outruns its bytes, against the bf16 matrix peak.  `configs`
carries every workload of the benchmark's configuration list (median step time, per-kernel durations and roofline
fractions, counter traffic from profiles/), each timed like the headline over `--config-steps` steps.
`sketch` times the random-projection baseline of Sec. 4.6 (pamm_sketch + pamm_sketch_grad) on the headline workload at
the width that stores as much as PAMM's compression does, the same way, and gives both estimates' distance from the exact
product X^T dY (the shape of the paper's ablation, on synthetic data).
`cpu_baseline` is the fp64 oracle timed on this machine's host cores on the headline batch.  `exact_gemm` is the
plain X^T dY product (vendor BLAS through torch.matmul) on the same GPU, for scale only.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_PEAK_BF16_TFLOPS = 2500.0
FP32_MATRIX_PEAK_TFLOPS = 157.3


def algorithmic_bytes(w, piece_rows_overhead=0):
    """Bytes the method must move per kernel launch (inputs once, outputs once)."""
    s = 2 if w.dtype == "bf16" else 4
    b, n, m, k = w.b, w.n, w.m, w.k
    return {
        "k_score": b * n * s + 8 * b,                  # X once; f and alpha are written by k_finalize (8 B/token)
        "k_contract": b * m * s + 8 * b + k * m * 4,   # dY once, (f, alpha) per row, Btilde out
        "k_ctb": n * m * 4 + k * n * s + k * m * 4,    # dW out, C and Btilde in
    }


def algorithmic_flops(w):
    """Multiply-adds x 2 of the two matrix products of the path (App. J counts the same products)."""
    return {"k_score": 2.0 * w.b * w.k * w.n, "k_ctb": 2.0 * w.k * w.n * w.m}


def read_traffic(workload: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), from the committed summary."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    mt = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    return float(mt.group(1)) if mt else None


def kernel_table(w, per_kernel_us):
    """Per kernel: average duration, algorithmic rate against the HBM peak, matrix rate against the bf16 MFMA peak."""
    alg, flops = algorithmic_bytes(w), algorithmic_flops(w)
    peak_tf = MFMA_PEAK_BF16_TFLOPS if w.dtype == "bf16" else FP32_MATRIX_PEAK_TFLOPS
    out = {}
    for name, us in per_kernel_us.items():
        ent = {"avg_us": round(us, 2)}
        if name in alg:
            gbs = alg[name] / (us * 1e-6) / 1e9
            ent["algorithmic_bytes"] = alg[name]
            ent["algorithmic_GBps"] = round(gbs, 1)
            ent["frac_of_hbm_peak"] = round(gbs / HBM_PEAK_GBS, 4)
            ent["traffic"] = read_traffic(w.name, name)
        if name in flops:
            tf = flops[name] / (us * 1e-6) / 1e12
            ent["TFLOPs"] = round(tf, 1)
            ent["frac_of_matrix_peak"] = round(tf / peak_tf, 4)
            # which roof is nearer: the time the bytes need at the HBM peak against the time the flops need at the matrix peak
            ent["bound"] = "mfma" if flops[name] / (peak_tf * 1e12) > alg[name] / (HBM_PEAK_GBS * 1e9) else "hbm"
        elif name in alg:
            ent["bound"] = "hbm"
        out[name] = ent
    return out


def time_workload(torch, pamm, workloads, name, steps, warmup, nsets, eps=None, dw="f32", dw_transposed=False):
    """K timed steps of compress + grad on one workload.  Returns (record, tensors kept for the optional extra legs)."""
    w = workloads.WORKLOADS[name]
    X_cpu, dY_cpu = workloads.generate(w)
    Xs = [X_cpu.cuda() for _ in range(nsets)]
    dYs = [dY_cpu.cuda() for _ in range(nsets)]
    b, n, m, k = w.b, w.n, w.m, w.k
    dt = pamm.PAMM_BF16 if w.dtype == "bf16" else pamm.PAMM_F32
    out = pamm.Compressed(torch.empty(k, n, dtype=Xs[0].dtype, device="cuda"), torch.empty(b, dtype=torch.int32, device="cuda"),
                          torch.empty(b, dtype=torch.float32, device="cuda"))
    dw_kw = {}
    if dw != "f32" or dw_transposed:
        dw_kw = dict(out_dtype=torch.bfloat16 if dw == "bf16" else torch.float32, transposed=dw_transposed)
    dW = torch.empty((m, n) if dw_transposed else (n, m), dtype=dw_kw.get("out_dtype", torch.float32), device="cuda")
    ws_c = torch.empty(pamm.compress_workspace(b, n, k, dt), dtype=torch.uint8, device="cuda")
    ws_g = torch.empty(pamm.grad_workspace(b, n, k, m, dt), dtype=torch.uint8, device="cuda")

    def step(i):
        pamm.compress(Xs[i % nsets], k, seed=i, eps=eps, out=out, ws=ws_c)      # fresh generators every step, as in training (App. F)
        pamm.grad(out.C, out.f, out.alpha, dYs[i % nsets], eta=out.eta, out=dW, ws=ws_g, **dw_kw)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    # every step on its own (events on the current stream, which is the stream the kernels are launched on):
    # the median step, and the split between the two calls
    reps = max(1, min(steps, 100))
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(reps)]
    for i in range(reps):
        ev[i][0].record()
        pamm.compress(Xs[i % nsets], k, seed=i, eps=eps, out=out, ws=ws_c)
        ev[i][1].record()
        pamm.grad(out.C, out.f, out.alpha, dYs[i % nsets], eta=out.eta, out=dW, ws=ws_g, **dw_kw)
        ev[i][2].record()
    torch.cuda.synchronize()
    tcs = sorted(e[0].elapsed_time(e[1]) for e in ev)
    tgs = sorted(e[1].elapsed_time(e[2]) for e in ev)
    tot = sorted(e[0].elapsed_time(e[2]) for e in ev)
    med = lambda v: v[len(v) // 2]

    # per-kernel durations: the same K steps again with the library's event hooks on
    pamm.profile_begin()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    prof = pamm.profile_end()
    per_kernel_us = {kname: 1e3 * ms / cnt for kname, (ms, cnt) in prof.items()}
    launches = sum(cnt for _, cnt in prof.values()) / steps

    rec = {
        "workload": w.name, "b": b, "n": n, "m": m, "k": k, "dtype": w.dtype, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(med(tot), 4),
        "tokens_per_s": round(b / (ms_per_step * 1e-3), 1),
        "ms_compress": round(med(tcs), 4), "ms_grad": round(med(tgs), 4), "launches_per_step": round(launches, 2),
        "kernels": kernel_table(w, per_kernel_us),
    }
    return rec, dict(w=w, X_cpu=X_cpu, dY_cpu=dY_cpu, X=Xs[0], dY=dYs[0], per_kernel_us=per_kernel_us)


def time_sketch(torch, pamm, workloads, name, steps, warmup, nsets):
    """The random-projection baseline on one workload: K timed steps of sketch + sketch_grad at the memory-matched width,
    per-kernel durations, and the relative error of both estimates of X^T dY."""
    w = workloads.WORKLOADS[name]
    if w.dtype != "bf16":
        return None
    r = workloads.matched_sketch_width(w)
    if r > 128:            # wider than the library's widest sketch (k = 1024 at the 7B-shaped layer would need 264 columns)
        return None
    X_cpu, dY_cpu = workloads.generate(w)
    Xs = [X_cpu.cuda() for _ in range(nsets)]
    dYs = [dY_cpu.cuda() for _ in range(nsets)]
    Pt = workloads.sketch_directions(w, r).cuda()
    b, n, m, k = w.b, w.n, w.m, w.k
    S = torch.empty(b, r, dtype=Xs[0].dtype, device="cuda")
    dW = torch.empty(n, m, dtype=torch.float32, device="cuda")
    ws = torch.empty(pamm.sketch_grad_workspace(b, n, r, m, pamm.PAMM_BF16), dtype=torch.uint8, device="cuda")

    def step(i):
        pamm.sketch(Xs[i % nsets], Pt, out=S)
        pamm.sketch_grad(Pt, S, dYs[i % nsets], out=dW, ws=ws)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    pamm.profile_begin()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    prof = pamm.profile_end()
    per_kernel_us = {kname: 1e3 * ms / cnt for kname, (ms, cnt) in prof.items()}
    alg = {"k_sketch": b * n * 2 + b * r * 2, "k_sketch_contract": b * m * 2 + b * r * 2 + r * m * 4,
           "k_ctb": n * m * 4 + r * n * 2 + r * m * 4}
    kernels = {}
    for kname, us in per_kernel_us.items():
        ent = {"avg_us": round(us, 2)}
        if kname in alg:
            gbs = alg[kname] / (us * 1e-6) / 1e9
            ent.update(algorithmic_bytes=alg[kname], algorithmic_GBps=round(gbs, 1), frac_of_hbm_peak=round(gbs / HBM_PEAK_GBS, 4),
                       bound="hbm", traffic=read_traffic(w.name, kname))
        kernels[kname] = ent

    # how far both estimates are from the exact product, in relative Frobenius norm (fp32 product of the same inputs)
    exact = torch.matmul(Xs[0].float().t(), dYs[0].float())
    step(0)
    err_sketch = float((dW - exact).norm() / exact.norm())
    c = pamm.compress(Xs[0], k, seed=0)
    err_pamm = float((pamm.grad(c.C, c.f, c.alpha, dYs[0]) - exact).norm() / exact.norm())
    torch.cuda.synchronize()
    return {
        "workload": w.name, "r": r, "stored_numbers": {"sketch": b * r, "pamm": k * n + 2 * b},
        "ms_per_step": round(ms_per_step, 4), "tokens_per_s": round(b / (ms_per_step * 1e-3), 1),
        "launches_per_step": round(sum(cnt for _, cnt in prof.values()) / steps, 2), "kernels": kernels,
        "rel_error_vs_exact": {"sketch": round(err_sketch, 4), "pamm": round(err_pamm, 4)},
        "what": "S = X P, dW = P S^T dY with P Gaussian (Sec. 4.6), same inputs, same rotation of input copies as the headline",
    }


ALL_WORKLOADS = ["tiny", "llama60m", "llama350m", "llama1b", "llama7b_k32", "llama7b_k256", "llama7b_k1024"]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama1b")
    ap.add_argument("--sets", type=int, default=2,
                    help="copies of (X, dY) in HBM that consecutive steps rotate through, so that no input survives in the "
                         "256 MiB Infinity Cache from one step to the next (1 = every step re-reads the same buffers)")
    ap.add_argument("--eps", type=float, default=None,
                    help="time the path with the neighbourhood condition of Eq. 2 at this tolerance (default: none, eps = infinity)")
    ap.add_argument("--dw", choices=["f32", "bf16"], default="f32",
                    help="element type of the weight gradient (default fp32, the configuration the metric is quoted on)")
    ap.add_argument("--dw-transposed", action="store_true", help="write the weight gradient as m x n instead of n x m")
    ap.add_argument("--layer", action="store_true",
                    help="also time the forward + backward pass of the linear layer of Alg. 2-3 (exact products through the "
                         "vendor BLAS) against the same layer with the exact weight gradient; adds a \"layer\" object")
    ap.add_argument("--no-configs", action="store_true", help="time the headline workload only (no \"configs\" array)")
    ap.add_argument("--config-steps", type=int, default=100, help="timed steps for each entry of the \"configs\" array")
    ap.add_argument("--no-sketch", action="store_true", help="do not time the random-projection baseline (no \"sketch\" object)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-exact-gemm", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (the reference reading for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the PAMM path has no CPU fallback", file=sys.stderr)
        return 3
    from paper_2506_02939_amd import pamm, workloads

    nsets = max(1, args.sets)
    rec, kept = time_workload(torch, pamm, workloads, args.workload, args.steps, args.warmup, nsets, eps=args.eps, dw=args.dw,
                              dw_transposed=args.dw_transposed)
    w, X, dY, X_cpu, dY_cpu = kept["w"], kept["X"], kept["dY"], kept["X_cpu"], kept["dY_cpu"]
    b, n, m, k = w.b, w.n, w.m, w.k
    kernels = rec["kernels"]

    dom = "k_contract"
    roofline = {
        "kernel": dom, "bound": "hbm", "achieved": kernels[dom]["algorithmic_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": kernels[dom]["frac_of_hbm_peak"], "traffic": kernels[dom]["traffic"],
        "algorithmic_bytes_per_launch": kernels[dom]["algorithmic_bytes"], "avg_launch_us": kernels[dom]["avg_us"],
    }
    hot = {name: kernels[name] for name in ("k_score", "k_contract", "k_ctb") if name in kernels}

    result = {
        "metric": "PAMM compress+grad tokens/s", "value": rec["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "b": b, "n": n, "m": m, "k": k, "dtype": w.dtype,
                   "recipe": f"{w.centres} centres, sigma {w.sigma}, {w.structure}, pad {w.pad_frac}",
                   "input_sets_rotated": nsets, "eps": args.eps,
                   "dW": args.dw + (" m x n" if args.dw_transposed else " n x m"),
                   "Btilde": "bf16 operand of the C^T Btilde product (rounded once from fp32 sums)" if w.dtype == "bf16" else "fp32"},
        "ms_per_step_median": rec["ms_per_step_median"],
        "ms_compress": rec["ms_compress"], "ms_grad": rec["ms_grad"], "launches_per_step": rec["launches_per_step"],
        "roofline": roofline,
        "roofline_kernels": hot,
        "min_hbm_bound_frac": min((v["frac_of_hbm_peak"] for v in hot.values() if v.get("bound") == "hbm"), default=None),
        "kernels": kernels,
    }
    del kept

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["calibrate_copy_bytes"] = 1 << 30
        del src, dst

    if not args.no_exact_gemm:
        Xt = X.t().contiguous()
        for _ in range(3):
            torch.matmul(Xt, dY)
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        reps_g = 20
        for _ in range(reps_g):
            torch.matmul(Xt, dY)
        torch.cuda.synchronize()
        gms = (time.perf_counter() - g0) * 1e3 / reps_g
        result["exact_gemm"] = {"ms": round(gms, 4), "tokens_per_s": round(b / (gms * 1e-3), 1),
                                "TFLOPs": round(2.0 * b * n * m / (gms * 1e-3) / 1e12, 1), "kind": "torch.matmul(X^T, dY), same GPU"}

    if not args.no_sketch:
        torch.cuda.empty_cache()
        sk = time_sketch(torch, pamm, workloads, w.name, min(args.steps, args.config_steps), min(args.warmup, 10), nsets)
        if sk is not None:
            result["sketch"] = sk

    if args.layer:
        from paper_2506_02939_amd import linear

        Xl = X.detach().clone().requires_grad_(True)
        Wl = (torch.randn(n, m, device="cuda") / n ** 0.5).to(X.dtype).requires_grad_(True)

        def layer_step(i, approx):
            Xl.grad = None
            Wl.grad = None
            Z = linear.pamm_linear(Xl, Wl, k=k, seed=i, eps=args.eps, overlap=approx == "overlap") if approx else torch.matmul(Xl, Wl)
            Z.backward(dY)

        layer = {}
        for approx in (True, "overlap", False):
            for i in range(3):
                layer_step(i, approx)
            torch.cuda.synchronize()
            l0 = time.perf_counter()
            reps_l = 10
            for i in range(reps_l):
                layer_step(i, approx)
            torch.cuda.synchronize()
            layer[{True: "ms_pamm", "overlap": "ms_pamm_overlapped", False: "ms_exact"}[approx]] = round((time.perf_counter() - l0) * 1e3 / reps_l, 4)
        layer["what"] = ("Z = X W, backward with dZ = dY: dX exact, dW by PAMM (ms_pamm; ms_pamm_overlapped: Compress and ApproxMM on a "
                         "second stream beside the GEMMs) or exact (ms_exact); GEMMs by torch.matmul")
        result["layer"] = layer
        del Xl, Wl

    if not args.no_cpu_baseline:
        from oracle import pamm_oracle

        pamm_oracle.build()
        best = None
        reps_cpu = 3
        for _ in range(reps_cpu):
            c0 = time.perf_counter()
            oc = pamm_oracle.compress(X_cpu, k, seed=0, eps=float("inf") if args.eps is None else args.eps)
            c1 = time.perf_counter()
            pamm_oracle.grad(oc.C, oc.f, oc.alpha, dY_cpu, beta=oc.beta)
            c2 = time.perf_counter()
            if best is None or c2 - c0 < best[0]:
                best = (c2 - c0, c1 - c0, c2 - c1)
        result["cpu_baseline"] = {
            "value": round(b / best[0], 1), "unit": "tokens/s", "cores": pamm_oracle.threads(), "kind": "oracle",
            "sample": f"the full {w.name} batch ({b} tokens), best of {reps_cpu} repetitions: "
                      f"compress {best[1]:.2f} s + grad {best[2]:.2f} s",
        }

    if not args.no_configs:
        # every workload of the configuration list, timed like the headline (no oracle leg: that runs once, above)
        configs = []
        for name in ALL_WORKLOADS:
            if name == w.name and args.eps is None and args.dw == "f32" and not args.dw_transposed:
                configs.append({key: rec[key] for key in rec})
                continue
            torch.cuda.empty_cache()
            r, kept_c = time_workload(torch, pamm, workloads, name, args.config_steps, min(args.warmup, 10), nsets)
            del kept_c
            configs.append(r)
        result["configs"] = configs

    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
