"""Host-side checks of bench.py's contract: it refuses more than one GPU with a message
(this build is single-GPU), and without a GPU it fails loudly instead of falling back to
a CPU path."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True,
                          text=True, timeout=300, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_no_silent_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        return                                  # on a GPU machine the bench itself is the check
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode != 0 and "no GPU" in r.stderr and r.stdout.strip() == ""
