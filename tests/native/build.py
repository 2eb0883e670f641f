"""Builds the torch-free test caller of the C-ABI (abi_roundtrip.cpp).  Test infrastructure: the
program links the CPU oracle as its checker, so this lives under tests/, not in the package."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "abi_roundtrip.cpp")
BIN = os.path.join(HERE, "abi_roundtrip")


def build(verbose: bool = False) -> str:
    """Needs paper_1910_04540_amd/libqsim.so and oracle/libqsim_ref.so to exist."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    pkg = os.path.join(ROOT, "paper_1910_04540_amd")
    oracle = os.path.join(ROOT, "oracle")
    cmd = [hipcc, "-O2", "-std=c++17", f"-I{os.path.join(ROOT, 'include')}", f"-I{oracle}", SRC,
           f"-L{pkg}", "-lqsim", f"-L{oracle}", "-lqsim_ref",
           "-Wl,-rpath,$ORIGIN/../../paper_1910_04540_amd", "-Wl,-rpath,$ORIGIN/../../oracle", "-o", BIN]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return BIN


if __name__ == "__main__":
    print(build(verbose=True))
