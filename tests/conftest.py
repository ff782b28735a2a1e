import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle


@pytest.fixture(scope="session")
def gpu():
    """torch on cuda:0 with the HIP library loaded; the tests using it are marked gpu."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2311_09550_amd as w4a8
    w4a8.lib()  # raises if the HIP library is missing: there is no fallback to test
    torch.cuda.set_device(0)
    return torch
