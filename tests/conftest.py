import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu_lib():
    """The HIP library binding; fails loudly if the extension or the GPU is missing."""
    import torch
    if not torch.cuda.is_available():
        pytest.fail("a test marked gpu ran on a box with no GPU")
    import paper_1803_09926_amd as dw
    dw.load()  # raises if libdwconv.so is not built
    return dw
