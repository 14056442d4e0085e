import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def lib():
    """The loaded HIP library's Python binding (built first only if no library is there yet).
    There is no fallback: if it cannot be built or loaded, every GPU test errors out."""
    from paper_2412_20501_amd.build import ensure_built
    ensure_built()
    import paper_2412_20501_amd as tr
    return tr
