import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The tests load the libraries that are built.  One that is missing, or that was built from other sources than
    # the ones on disk (each library carries a digest of its sources), is rebuilt here first; hipcc cross-compiles
    # for gfx950 without a GPU.  A stale library is never tested: if the rebuild fails, so does the session.
    from paper_2003_00532_amd import build as hip_build
    from oracle import build as oracle_build
    for mod, what in ((hip_build, "HIP library"), (oracle_build, "CPU oracle")):
        if mod.is_stale():
            try:
                mod.build()
            except Exception as e:   # noqa: BLE001
                raise pytest.UsageError("%s at %s is out of date and could not be rebuilt: %s" % (what, mod.LIB, e))
            if mod.is_stale():
                raise pytest.UsageError("%s at %s is still out of date after a rebuild" % (what, mod.LIB))


@pytest.fixture(scope="session")
def gpu_device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    return torch.device("cuda:0")
