"""CPU-only checks of bench.py's command line: it refuses more than one GPU with a message that says
why, and without a GPU it fails loudly instead of timing anything else."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          cwd=ROOT, timeout=300)


def test_more_than_one_gpu_is_refused():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_without_a_gpu_nothing_is_timed():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    r = _run("--steps", "2", "--warmup", "1")
    assert r.returncode != 0
    assert "no GPU" in r.stderr and r.stdout.strip() == ""
