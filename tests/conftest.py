import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load what is built; they build only if nothing is
    lib = os.path.join(ROOT, "paper_2404_16109_amd", "libzkmi.so")
    if not os.path.exists(lib):
        from paper_2404_16109_amd import build as hip_build
        hip_build.build()


@pytest.fixture(scope="session")
def orc():
    """The CPU oracle's ctypes binding (builds liboracle.so on first use)."""
    from oracle import pyoracle
    pyoracle.lib()
    return pyoracle
