"""bench.py's command line contract that can be checked without a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def _run(*args):
    return subprocess.run([sys.executable, BENCH, *args], capture_output=True, text=True, timeout=300, cwd=ROOT)


@pytest.mark.parametrize("n", ["2", "8", "0"])
def test_more_than_one_gpu_is_refused_with_a_message(n):
    r = _run("--gpus", n)
    assert r.returncode == 2
    assert "ONE GPU" in (r.stdout + r.stderr)
    assert "{" not in r.stdout                      # no result line


def test_without_a_gpu_the_bench_fails_loudly_and_never_falls_back():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible here")
    r = _run()
    assert r.returncode != 0
    assert "no CPU fallback" in (r.stdout + r.stderr)
    assert "{" not in r.stdout
