"""The command-line entry points refuse loudly what they cannot do: more than one GPU, and (on a
machine without a GPU) running at all; nothing falls back to the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, *args], cwd=ROOT, capture_output=True, text=True, timeout=300)


def test_bench_refuses_more_than_one_gpu():
    r = _run("bench.py", "--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "one GPU" in r.stderr + r.stdout
    assert "{" not in r.stdout                       # no result line


def _gpu_here():
    torch = pytest.importorskip("torch")
    return torch.cuda.is_available()


@pytest.mark.parametrize("args", [("bench.py",), ("-m", "paper_1910_04540_amd.sweep"),
                                  ("-m", "paper_1910_04540_amd.tuning_scans", "--channel-shapes")])
def test_no_gpu_no_result(args):
    if _gpu_here():
        pytest.skip("this machine has a GPU")
    r = _run(*args)
    assert r.returncode != 0
    assert "GPU" in r.stderr + r.stdout
    assert "{" not in r.stdout
