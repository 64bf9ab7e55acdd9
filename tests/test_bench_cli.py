"""bench.py's command line where no GPU is needed to tell: more than one GPU is
refused with a message, and without a GPU there is no result line at all (no CPU
path stands in for the kernels)."""
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300, cwd=ROOT)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stdout + r.stderr
    assert "{" not in r.stdout


@pytest.mark.skipif(torch.cuda.is_available(), reason="only where there is no GPU")
def test_no_gpu_no_number():
    r = run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "needs a GPU" in r.stderr
    assert "{" not in r.stdout
