"""Host-only checks of bench.py's command line: what it refuses, and that it
never falls back to anything when there is no GPU."""
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2
    assert "exactly one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.skipif(torch.cuda.is_available(), reason="needs a machine without a GPU")
def test_without_a_gpu_it_fails_loudly_and_prints_no_result():
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode == 1
    assert "no GPU visible" in r.stderr and r.stdout.strip() == ""
