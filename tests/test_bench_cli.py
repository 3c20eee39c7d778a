"""bench.py's command line without a GPU: more than one GPU is refused with a message, and a machine without
a GPU gets an error, never a CPU fallback."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          cwd=ROOT, timeout=300)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2")
    assert r.returncode == 2 and "--gpus must be 1" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_means_an_error_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        import pytest
        pytest.skip("a GPU is present")
    r = run("--steps", "1", "--warmup", "0", "--workload", "tiny")
    assert r.returncode == 3 and "no CPU fallback" in r.stderr and r.stdout.strip() == ""
