import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the in-tree libraries; compile them only when nothing has been built yet
    from paper_2507_19906_amd import build as _build
    if not (os.path.exists(_build.LIB_PATH) and os.path.exists(_build.PROBES_PATH)):
        _build.build()


@pytest.fixture(scope="session")
def have_gpu():
    import torch
    return torch.cuda.is_available()
