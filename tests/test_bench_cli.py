"""bench.py's contract on a box without a GPU: more than one GPU is refused with a message that says
why, and without a GPU the benchmark stops loudly instead of falling back to anything (CPU only)."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=dict(os.environ, **(env or {})), timeout=300)


def test_more_than_one_gpu_is_refused():
    r = run("--gpus", "2")
    assert r.returncode != 0 and "ONE GPU" in r.stderr
    r = run(env={"WORLD_SIZE": "2"})
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_no_gpu_no_fallback():
    if torch.cuda.is_available():
        return
    r = run()
    assert r.returncode != 0 and "no CPU fallback" in r.stderr
    assert "{" not in r.stdout                      # no result line is printed
