import os
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
for path in (ROOT, HERE):
    if path not in sys.path:
        sys.path.insert(0, path)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu():
    """(library binding, device helpers, torch) for the tests marked gpu; the library must be built."""
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    import paper_2604_18655_amd as lib
    from paper_2604_18655_amd import device
    lib.load_library()
    return lib, device, torch
