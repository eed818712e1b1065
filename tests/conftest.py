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
    """torch device for GPU tests; fails (not skips) when the HIP library cannot be used."""
    import torch
    assert torch.cuda.is_available(), "GPU test selected but no GPU is visible"
    from paper_2207_00032_amd import binding
    binding.load()  # raises if libsbi_gemm.so is missing: no silent fallback
    return torch.device("cuda:0")
