import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _ensure_hip_library():
    """Tests load the library that is built; only if there is none do they build it (hipcc cross-compiles)."""
    from paper_2312_00839_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2312_00839_amd import build as hip_build
        hip_build.build()


def pytest_configure(config):
    _ensure_hip_library()
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: CPU test that takes more than a few seconds")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle
