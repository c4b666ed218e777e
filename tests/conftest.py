import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def ess_lib():
    """The loaded C-ABI library; GPU tests must run on it and nothing else."""
    import torch
    from paper_2512_10576_amd import binding
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return binding.load()
