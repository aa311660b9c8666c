"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr + r.stdout and "{" not in r.stdout      # no result line


def test_without_a_gpu_the_bench_fails_loudly():
    if torch.cuda.is_available():
        return                                   # covered by the GPU runs
    r = run("--steps", "1", "--warmup", "0", "--no-cpu-baseline")
    assert r.returncode != 0 and '"metric"' not in r.stdout             # no CPU fallback, no number
