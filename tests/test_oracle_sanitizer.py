"""The oracle's C source under the undefined-behaviour sanitizer (host code only): a build with
-fsanitize=undefined -fno-sanitize-recover=all must run the sampler, Compress (with and without the tolerance) and
ApproxMM over ordinary and degenerate inputs without a report.  Runs in a child process: a report aborts it.
"""
import os
import subprocess
import sys
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_ubsan(tmp_path):
    lib = tmp_path / "liboracle_ubsan.so"
    src = os.path.join(ROOT, "oracle", "pamm_oracle.c")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-shared",
                    "-fPIC", "-o", str(lib), src, "-lm"], check=True)
    script = textwrap.dedent(f"""
        import importlib.util, sys
        import numpy as np, torch
        spec = importlib.util.spec_from_file_location("oracle_ubsan", {os.path.join(ROOT, "oracle", "pamm_oracle.py")!r})
        o = importlib.util.module_from_spec(spec); sys.modules[spec.name] = o; spec.loader.exec_module(o)
        o._LIB = {str(lib)!r}; o._lib = None; o.build = lambda force=False: {str(lib)!r}
        g = np.random.default_rng(0)
        for b, n, m, k in [(1, 4, 4, 1), (7, 8, 12, 7), (300, 24, 10, 9), (1000, 40, 16, 64)]:
            for make in (lambda a: a.astype(np.float32), lambda a: torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)):
                X = g.standard_normal((b, n)); X[b // 2] = 0.0
                B = g.standard_normal((b, m))
                for eps in (float("inf"), 0.0, 0.4):
                    c = o.compress(make(X), k, seed=b, eps=eps)
                    o.grad(c.C, c.f, c.alpha, make(B), beta=c.beta)
        assert sorted(o.sample(64, 64, 2**64 - 1).tolist()) == list(range(64))
        o.sample(10**6, 5, 0)
        print("clean")
    """)
    r = subprocess.run([sys.executable, "-c", script], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0 and "clean" in r.stdout, r.stderr[-2000:]
    assert "runtime error" not in r.stderr
