"""Refusals that need no GPU: bench.py on more than one GPU or without a GPU, and the binding without its library."""
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful on a machine without a GPU")
def test_no_gpu_means_no_result_rather_than_a_cpu_fallback():
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "no CPU fallback" in r.stderr and r.stdout.strip() == ""


def test_binding_without_the_library_fails_loudly(tmp_path):
    """A copy of the package without libpamm.so cannot be imported: no silent fallback of any kind."""
    pkg = tmp_path / "paper_2506_02939_amd"
    pkg.mkdir()
    src = os.path.join(ROOT, "paper_2506_02939_amd")
    for name in ("__init__.py", "pamm.py"):
        (pkg / name).write_text(open(os.path.join(src, name)).read())
    r = subprocess.run([sys.executable, "-c", "import paper_2506_02939_amd.pamm"], cwd=str(tmp_path), capture_output=True,
                       text=True, timeout=300, env={**os.environ, "PYTHONPATH": str(tmp_path)})
    assert r.returncode != 0
    assert "ImportError" in r.stderr and "no CPU fallback" in r.stderr
