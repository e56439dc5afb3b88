import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# PyTorch ships its own copy of the HIP runtime.  Tests that use torch for device buffers need the library
# under test to bind to that same copy, which happens when torch is loaded first; a test order (or -k
# selection) that loads the library first would leave torch unable to see the GPU afterwards.
try:
    import torch  # noqa: F401
except ImportError:  # CPU-only environments without torch still run the oracle and ABI tests
    pass


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_oracle():
    from oracle import Oracle, Params
    import workloads as wl
    return Oracle(Params(*wl.WORKLOADS[0].param_tuple()))
