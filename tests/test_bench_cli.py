"""The benchmark's command line where no GPU is needed: more than one GPU is refused with a message, and
without a GPU it says so instead of falling back to anything."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused():
    res = run("--gpus", "2")
    assert res.returncode == 2
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_no_gpu_no_fallback():
    import torch
    if torch.cuda.is_available():
        import pytest
        pytest.skip("a GPU is visible here")
    res = run("--steps", "1", "--warmup", "0")
    assert res.returncode == 2
    assert "no GPU" in res.stderr and res.stdout.strip() == ""
