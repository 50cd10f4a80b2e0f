import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(scope="session")
def torch_cuda():
    """torch with a GPU and the built library loaded; GPU tests fail (not skip) without them."""
    import torch
    from paper_2603_28768_amd import binding
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    assert os.path.exists(binding.LIB_PATH), "libcraft.so has not been built"
    binding.lib()
    return torch
