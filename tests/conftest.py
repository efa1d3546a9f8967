import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """The tests load the in-tree library; build it (hipcc cross-compiles without a GPU) when a fresh
    checkout has none.  A build that exists is used as it is."""
    lib = os.path.join(ROOT, "paper_2405_18328_amd", "libgpws.so")
    if not os.path.exists(lib):
        from paper_2405_18328_amd.build import build_library
        build_library(verbose=False)
