import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _built_helpers():
    """Host-side helper libraries (input generator, C oracle) are built on demand; HIP is not."""
    import pv_inputs
    from oracle import build as obuild
    pv_inputs.build(force=False)
    obuild.build(force=False)
