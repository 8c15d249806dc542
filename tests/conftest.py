import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # Load what is built; build only if nothing is (hipcc cross-compiles without a GPU).
    from paper_2604_24088_amd import build as hip_build
    hip_build.ensure_built()


@pytest.fixture(scope="session")
def oracle():
    from oracle import taco_ref
    taco_ref.lib()
    return taco_ref
