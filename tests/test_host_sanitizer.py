"""The host side of libpamm under the address and undefined-behaviour sanitizers, on the CPU: tests/host_sanitize.cpp
pulls in csrc/api.cpp and csrc/pamm_plan.h (sampler, launch planners, workspace arithmetic, every argument check of
the entry points) and runs them over ordinary, extreme and invalid arguments.  A report aborts the child process."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "host_sanitize"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-D__HIP_PLATFORM_AMD__", f"-I{ROCM}/include", os.path.join(ROOT, "tests", "host_sanitize.cpp"), "-o", str(exe),
           f"-L{ROCM}/lib", "-lamdhip64", f"-Wl,-rpath,{ROCM}/lib"]
    subprocess.run(cmd, check=True, timeout=600)
    # the HIP runtime the binary links against is not instrumented and keeps process-lifetime allocations
    env = {**os.environ, "ASAN_OPTIONS": "detect_leaks=0"}
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0 and r.stdout.strip() == "clean", (r.stdout[-500:], r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
