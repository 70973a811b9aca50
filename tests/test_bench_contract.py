"""bench.py's command-line contract, as far as it can be checked without a GPU: more than one GPU
is refused with a message, and without a GPU the script stops instead of computing on the CPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_means_no_result():
    import torch
    if torch.cuda.is_available():
        return                      # on a GPU machine the bench itself is the test
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode == 3
    assert "no CPU fallback" in r.stderr and r.stdout.strip() == ""
