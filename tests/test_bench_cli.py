"""bench.py on a machine without a GPU: the one-GPU contract and the failure without a device
are reported as errors, never papered over by a CPU path."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, env=env,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""
    r = run(env=dict(os.environ, WORLD_SIZE="8"))
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_no_gpu_no_number():
    import torch
    if torch.cuda.is_available():
        return                                   # on a GPU machine the real benchmark would run
    r = run("--steps", "1", "--no-cpu")
    assert r.returncode == 1 and "no CPU fallback" in r.stderr and r.stdout == ""
