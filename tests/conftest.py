import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def fftconv_lib_path():
    """Path of the built HIP library; builds it once if absent (hipcc cross-compiles without a GPU)."""
    from paper_1312_5851_amd import build as _build
    path = _build.lib_path()
    if not os.path.exists(path):
        _build.build_library()
    return path
