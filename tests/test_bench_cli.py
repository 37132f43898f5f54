"""Command-line contract of bench.py that needs no GPU: one GPU only, and no silent fallback."""
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = run("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr + p.stdout
    assert "{" not in p.stdout  # no result line


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the behaviour on a machine without a GPU")
def test_without_a_gpu_the_bench_fails_instead_of_falling_back():
    p = run("--steps", "1", "--warmup", "0", "--no-cpu-baseline", "--no-extras")
    assert p.returncode != 0
    assert '"metric"' not in p.stdout
