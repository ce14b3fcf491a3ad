"""bench.py's command line on a machine without a GPU: it must refuse more than one GPU with a message, and must
not pretend to measure when no GPU is visible.  CPU only."""
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout) and not r.stdout.strip().startswith("{")


@pytest.mark.skipif(torch.cuda.is_available(), reason="needs a machine without a GPU")
def test_without_a_gpu_nothing_is_reported():
    r = run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0 and "no GPU" in (r.stderr + r.stdout) and "{" not in r.stdout


def test_unknown_workload_is_an_argument_error():
    r = run("--workload", "nonsense")
    assert r.returncode == 2
