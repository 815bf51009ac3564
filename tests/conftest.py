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
    """The ctypes binding, loaded once; fails loudly if the HIP library is not built."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2601_17917_amd as sd
    sd.load_library()
    return sd
