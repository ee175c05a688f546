import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu():
    """The HIP library bound to cuda:0; fails loudly when either is missing."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2411_05309_amd as gv
    gv.load()          # raises if libgpuvm.so has not been built
    return gv


@pytest.fixture
def say(capsys):
    """Progress lines of a long test, printed past pytest's capture so that a
    watcher of the run sees that it is alive."""
    import time

    def _say(what):
        with capsys.disabled():
            print(f"\n[{time.strftime('%H:%M:%S')}] {what}", end="", flush=True)
    return _say
