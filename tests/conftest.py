import os
import sys
import time

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def lib():
    """The HIP library's Python binding; GPU tests fail loudly if the extension is missing."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    import paper_2202_09512_amd as nn
    nn.load()          # raises if the shared library was not built
    return nn


@pytest.fixture
def progress(capsys):
    """A print that reaches the terminal while the test still runs (output capture switched off for the line): the
    full-size tests take minutes and say which step they are at."""
    def say(msg):
        with capsys.disabled():
            print(f"\n[{time.strftime('%H:%M:%S')}] {msg}", end="", flush=True)
    return say
