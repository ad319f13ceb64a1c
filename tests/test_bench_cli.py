"""bench.py's command line without a GPU: more than one GPU is refused with a
message, and a machine without a GPU is reported rather than worked around."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args],
                          capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused():
    out = run("--gpus", "2")
    assert out.returncode == 2
    assert "ONE GPU" in out.stderr and not out.stdout.strip()


def test_no_gpu_no_number():
    import torch
    if torch.cuda.is_available():
        return                                  # on a GPU machine the real bench covers this path
    out = run("--steps", "1", "--no-cpu-baseline")
    assert out.returncode == 2
    assert "needs a GPU" in out.stderr and not out.stdout.strip()
