import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _ensure_library():
    """Tests load the library that is built; it is built here only when there is none, or when the one that is
    there was built from other sources than the tree holds now (the binding refuses to load such a library)."""
    from paper_2412_18106_amd import build as _build
    if not _build.is_current():
        _build.build()


_ensure_library()
