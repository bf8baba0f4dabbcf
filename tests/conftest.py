import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_collection_modifyitems(config, items):
    """GPU tests must fail loudly when selected without a GPU; they are only skipped when not selected."""
    return


@pytest.fixture(scope="session")
def gpu_lib():
    """The built HIP library through its ctypes binding; a missing library or GPU is an error, not a skip."""
    import torch
    from paper_2605_27740_amd import binding
    assert torch.cuda.is_available(), "GPU tests were selected but no GPU is visible"
    return binding.load()
