"""bench.py's command line on a machine without a GPU: more than one GPU is refused with a message,
and without a device the run stops before anything is measured (there is no CPU fallback)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          cwd=ROOT, timeout=300)


def test_more_than_one_gpu_is_refused():
    r = _run("--gpus", "2")
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        return                      # on a GPU machine the bench itself is run by the driver
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode == 2
    assert "no GPU" in r.stderr and r.stdout.strip() == ""
