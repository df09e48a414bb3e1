import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle.build()
    return oracle


def _gpu_ok() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


@pytest.fixture(scope="session")
def lantern_gpu():
    """The HIP library's Python binding, on a box that has a GPU."""
    if not _gpu_ok():
        pytest.skip("no GPU in this container")
    import paper_2410_03355_amd as lantern
    lantern.load()  # raises if the extension is missing: no CPU fallback exists
    return lantern
