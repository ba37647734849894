import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _ensure_library():
    """Tests load the library that is built; build it only when nothing is there."""
    lib = os.path.join(ROOT, "paper_2412_18106_amd", "libxyattn.so")
    if not os.path.exists(lib):
        from paper_2412_18106_amd import build as _build
        _build.build()


_ensure_library()
