import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # load what is built; build only if nothing is (hipcc cross-compiles without a GPU)
    import paper_2207_12000_amd as gp
    if not os.path.exists(gp.LIB_PATH):
        from paper_2207_12000_amd import build as libbuild
        libbuild.build()


def has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


@pytest.fixture(scope="session")
def gpu_or_skip():
    if not has_gpu():
        pytest.skip("no GPU in this environment")
