import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _native_library():
    """Use the library that is built; build it only if there is none."""
    from paper_1811_00206_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_1811_00206_amd.build import build_library
        build_library()
    return binding.load_library()
