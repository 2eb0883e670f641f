import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: exhaustive sweeps, opt-in with QSIM_EXHAUSTIVE=1")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(scope="session", autouse=True)
def _built_libraries():
    """Tests load what is built; they build only when nothing is there (a fresh checkout keeps no
    binaries).  The oracle's loader does the same for its own shared object."""
    lib = os.path.join(ROOT, "paper_1910_04540_amd", "libqsim.so")
    if not os.path.exists(lib):
        from paper_1910_04540_amd import build as hip_build
        hip_build.build()
