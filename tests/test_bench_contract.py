"""bench.py's command line contract, the parts that need no GPU: more than one GPU is refused with a message (this
build measures one GPU and has no inter-GPU path), and without a GPU the program says so instead of computing anything
on the CPU.  The JSON line itself is checked where a GPU is present (tests/test_gpu_bench_line.py)."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = _bench("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_without_a_gpu_nothing_is_computed():
    import torch

    if torch.cuda.is_available():
        return  # (on the GPU machine the line itself is tested)
    p = _bench("--steps", "1", "--warmup", "0")
    assert p.returncode != 0 and "no CPU fallback" in p.stderr and p.stdout.strip() == ""
