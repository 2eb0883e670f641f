"""The C-ABI without Python or PyTorch in the way: a small HIP program (tests/native/abi_roundtrip.cpp)
allocates device memory itself, calls the entry points on its own stream and compares every result
with the CPU oracle it links."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "native"))


def test_native_caller_of_the_c_abi():
    import build as native_build                     # tests/native/build.py

    if not os.path.exists(native_build.BIN):          # run what is built; build only when nothing is
        from oracle import qsim_ref
        qsim_ref.lib()
        native_build.build()
    run = subprocess.run([native_build.BIN], capture_output=True, text=True, timeout=120)
    print(run.stdout)
    print(run.stderr, file=sys.stderr)
    assert run.returncode == 0, run.stdout[-2000:]
    assert "all ok" in run.stdout
