import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP library)")
    # the CPU checker is plain C: make sure it is compiled before any test asks for it
    from oracle import build as oracle_build
    oracle_build.build()


@pytest.fixture(scope="session")
def qb():
    """The HIP library's Python binding; GPU tests only."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1909_05840_amd as pkg
    pkg.load_library()  # raises if libqbert.so is not built: never fall back to anything else
    return pkg
