import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the libraries that are built; only if one is missing altogether is it built here
    # (hipcc cross-compiles for gfx950 without a GPU)
    from paper_2003_00532_amd import build as hip_build
    from oracle import build as oracle_build
    if not os.path.exists(hip_build.LIB):
        hip_build.build()
    if not os.path.exists(oracle_build.LIB):
        oracle_build.build()


@pytest.fixture(scope="session")
def gpu_device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    return torch.device("cuda:0")
