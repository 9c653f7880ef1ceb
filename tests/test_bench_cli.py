"""bench.py's contract at the edges that need no GPU: more than one GPU is refused with a message, and without a GPU
the HIP path refuses to run (there is no CPU fallback to fall back to)."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_no_number():
    if torch.cuda.is_available():
        return                       # on a GPU machine the real run is what the driver checks
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode == 3
    assert "no GPU" in r.stderr and r.stdout.strip() == ""
