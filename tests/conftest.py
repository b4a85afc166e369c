import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    """The CPU oracle (compiled on first use)."""
    from oracle import fbsr_oracle
    fbsr_oracle.lib()
    return fbsr_oracle


@pytest.fixture(scope="session")
def fbsr():
    """The GPU library's Python binding; GPU tests fail loudly if it cannot load."""
    import paper_2504_20634_amd as pkg
    pkg.binding.lib()
    return pkg
