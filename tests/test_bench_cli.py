"""bench.py's command line on a machine without a GPU: more than one GPU is refused with a message (this
build runs on one GPU), and without a visible GPU the benchmark says so instead of falling back to anything."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_no_fallback():
    if torch.cuda.is_available():
        return                                        # on a GPU machine the benchmark itself is the test
    r = run("--steps", "1", "--warmup", "0")
    assert r.returncode == 1
    assert "no GPU" in r.stderr and r.stdout.strip() == ""
