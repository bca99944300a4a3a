import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _native_libs_present():
    """CPU-side shared objects are built on demand; the GPU library is never built here."""
    from paper_2307_05740_amd import _build
    if not os.path.exists(_build.SYNTH_LIB):
        _build.build_synth()
    if not os.path.exists(_build.ORACLE_LIB):
        _build.build_oracle()
