#!/usr/bin/env python3
"""Benchmark of the PAMM hot path on one MI355X: one step = pamm_compress + pamm_grad over one synthetic batch.

Prints ONE JSON line.  `value` is tokens/s = b / (t_compress + t_grad) with X and dY resident in HBM before the
timed region; consecutive steps rotate through `--sets` copies of the inputs so that a step finds none of its
inputs in the Infinity Cache.  `roofline` covers the dominant kernel (k_contract, the single pass over dY): algorithmic bytes per
launch divided by its mean duration, the latter measured here with HIP events on the launch stream (the library's
own per-kernel event hooks) over a second run of the same K steps.  `cpu_baseline` is the fp64 oracle timed on
this machine's host cores on the same batch.  `exact_gemm` is the plain X^T dY product (vendor BLAS through
torch.matmul) on the same GPU, for scale only.
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


def algorithmic_bytes(w, piece_rows_overhead=0):
    """Bytes the method must move per kernel launch (inputs once, outputs once)."""
    s = 2 if w.dtype == "bf16" else 4
    b, n, m, k = w.b, w.n, w.m, w.k
    return {
        "k_score": b * n * s + 8 * b,                  # X once; f and alpha are written by k_finalize (8 B/token)
        "k_contract": b * m * s + 8 * b + k * m * 4,   # dY once, (f, alpha) per row, Btilde out
        "k_ctb": n * m * 4 + k * n * s + k * m * 4,    # dW out, C and Btilde in
    }


def read_traffic(workload: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), from the committed summary."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    mt = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    return float(mt.group(1)) if mt else None


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

    w = workloads.WORKLOADS[args.workload]
    X_cpu, dY_cpu = workloads.generate(w)
    nsets = max(1, args.sets)
    Xs = [X_cpu.cuda() for _ in range(nsets)]
    dYs = [dY_cpu.cuda() for _ in range(nsets)]
    X, dY = Xs[0], dYs[0]
    b, n, m, k = w.b, w.n, w.m, w.k
    dt = pamm.PAMM_BF16 if w.dtype == "bf16" else pamm.PAMM_F32

    out = pamm.Compressed(torch.empty(k, n, dtype=X.dtype, device="cuda"), torch.empty(b, dtype=torch.int32, device="cuda"),
                          torch.empty(b, dtype=torch.float32, device="cuda"))
    dw_kw = {}
    if args.dw != "f32" or args.dw_transposed:
        dw_kw = dict(out_dtype=torch.bfloat16 if args.dw == "bf16" else torch.float32, transposed=args.dw_transposed)
    dW = torch.empty((m, n) if args.dw_transposed else (n, m), dtype=dw_kw.get("out_dtype", torch.float32), device="cuda")
    ws_c = torch.empty(pamm.compress_workspace(b, n, k, dt), dtype=torch.uint8, device="cuda")
    ws_g = torch.empty(pamm.grad_workspace(b, n, k, m, dt), dtype=torch.uint8, device="cuda")

    def step(i):
        pamm.compress(Xs[i % nsets], k, seed=i, eps=args.eps, out=out, ws=ws_c)      # fresh generators every step, as in training (App. F)
        pamm.grad(out.C, out.f, out.alpha, dYs[i % nsets], eta=out.eta, out=dW, ws=ws_g, **dw_kw)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # separate timing of the two calls (events on the current stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    tc = tg = 0.0
    reps = max(1, min(args.steps, 50))
    for i in range(reps):
        ev[0].record()
        pamm.compress(Xs[i % nsets], k, seed=i, eps=args.eps, out=out, ws=ws_c)
        ev[1].record()
        pamm.grad(out.C, out.f, out.alpha, dYs[i % nsets], eta=out.eta, out=dW, ws=ws_g, **dw_kw)
        ev[2].record()
        torch.cuda.synchronize()
        tc += ev[0].elapsed_time(ev[1])
        tg += ev[1].elapsed_time(ev[2])
    tc, tg = tc / reps, tg / reps

    # per-kernel durations: the same K steps again with the library's event hooks on
    pamm.profile_begin()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    prof = pamm.profile_end()
    per_kernel_us = {name: 1e3 * ms / cnt for name, (ms, cnt) in prof.items()}

    alg = algorithmic_bytes(w)
    dom = "k_contract"
    dur_s = per_kernel_us[dom] * 1e-6
    achieved = alg[dom] / dur_s / 1e9
    roofline = {
        "kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic(w.name, dom),
        "algorithmic_bytes_per_launch": alg[dom], "avg_launch_us": round(per_kernel_us[dom], 2),
    }
    kernels = {}
    for name, us in per_kernel_us.items():
        ent = {"avg_us": round(us, 2)}
        if name in alg:
            ent["algorithmic_GBps"] = round(alg[name] / (us * 1e-6) / 1e9, 1)
            ent["frac_of_hbm_peak"] = round(alg[name] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        if name == "k_score":
            ent["TFLOPs"] = round(2.0 * b * k * n / (us * 1e-6) / 1e12, 1)
        if name == "k_ctb":
            ent["TFLOPs"] = round(2.0 * k * n * m / (us * 1e-6) / 1e12, 1)
        kernels[name] = ent

    result = {
        "metric": "PAMM compress+grad tokens/s", "value": round(b / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "b": b, "n": n, "m": m, "k": k, "dtype": w.dtype,
                   "recipe": f"{w.centres} centres, sigma {w.sigma}, {w.structure}, pad {w.pad_frac}",
                   "input_sets_rotated": nsets, "eps": args.eps,
                   "dW": args.dw + (" m x n" if args.dw_transposed else " n x m")},
        "ms_compress": round(tc, 4), "ms_grad": round(tg, 4),
        "roofline": roofline,
        "kernels": kernels,
    }

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

    if args.layer:
        from paper_2506_02939_amd import linear

        Xl = X.detach().clone().requires_grad_(True)
        Wl = (torch.randn(n, m, device="cuda") / n ** 0.5).to(X.dtype).requires_grad_(True)

        def layer_step(i, approx):
            Xl.grad = None
            Wl.grad = None
            Z = linear.pamm_linear(Xl, Wl, k=k, seed=i, eps=args.eps) if approx else torch.matmul(Xl, Wl)
            Z.backward(dY)

        layer = {}
        for approx in (True, False):
            for i in range(3):
                layer_step(i, approx)
            torch.cuda.synchronize()
            l0 = time.perf_counter()
            reps_l = 10
            for i in range(reps_l):
                layer_step(i, approx)
            torch.cuda.synchronize()
            layer["ms_pamm" if approx else "ms_exact"] = round((time.perf_counter() - l0) * 1e3 / reps_l, 4)
        layer["what"] = "Z = X W, backward with dZ = dY: dX exact, dW by PAMM (ms_pamm) or exact (ms_exact); GEMMs by torch.matmul"
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

    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
