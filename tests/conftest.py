import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# Workloads whose candidates all place alike would be sent to the shared-placement kernel by Evaluator.for_workload;
# the tests of the other kernels keep them where they were, tests/test_gpu_shared_placement.py switches it back on.
os.environ.setdefault("DAGSCHED_NO_SHARED_PLACEMENT", "1")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu_lib():
    """The HIP library through its Python binding; fails loudly when it or the GPU is missing."""
    import torch
    if not torch.cuda.is_available():
        pytest.fail("a test marked gpu was run without a GPU")
    from paper_2503_09357_amd import dagsched
    dagsched.load()
    return dagsched
