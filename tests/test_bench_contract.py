"""bench.py on a box without the requested resources: more than one GPU is refused
with a message (this build is single-GPU by construction), and without any GPU the
benchmark stops instead of falling back to a CPU path."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + args, cwd=ROOT, env=e,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)


def test_more_than_one_gpu_is_refused():
    r = _run(["--gpus", "2", "--steps", "1", "--warmup", "0"])
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and not r.stdout.strip()


def test_world_size_above_one_is_refused():
    r = _run(["--steps", "1", "--warmup", "0"], env={"WORLD_SIZE": "2"})
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        import pytest
        pytest.skip("a GPU is visible")
    r = _run(["--steps", "1", "--warmup", "0"])
    assert r.returncode != 0
    assert "no GPU" in r.stderr and not r.stdout.strip()
