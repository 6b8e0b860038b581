import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as O
    O.build_oracle()
    return O


@pytest.fixture(scope="session")
def env(oracle):
    """(torch, binding, oracle) for the GPU tests: the HIP library must load and a GPU be there."""
    import torch
    from paper_2305_04359_amd import binding as A
    assert torch.cuda.is_available(), "these tests need the GPU"
    A.lib()
    return torch, A, oracle
