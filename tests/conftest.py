import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (run with -m gpu on the GPU box)")


def pytest_sessionstart(session):
    """The tests load the built library; only when none is there do they build it (hipcc
    cross-compiles without a GPU).  After a change to a source, build before running the tests."""
    from paper_1606_08495_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):
        hip_build.build()
