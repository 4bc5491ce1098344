import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# Workloads whose candidates all place alike are sent to the shared-placement kernel by Evaluator.for_workload.  The
# tests written for the other kernels (tests/test_gpu_parity.py, tests/test_gpu_search.py) ask, per test module and
# through dagsched_shape_t.ignore_shared_placement, to keep such workloads on those kernels; the full-size test of
# the five configurations runs both ways, and tests/test_gpu_shared_placement.py never switches the hint off.
RING_TEST_MODULES = ("test_gpu_parity", "test_gpu_search", "test_gpu_channels")


@pytest.fixture(autouse=True)
def _ring_kernel_modules(request):
    if request.module.__name__ in RING_TEST_MODULES:
        from paper_2503_09357_amd import dagsched as ds
        with ds.shape_defaults(ignore_shared_placement=1):
            yield
    else:
        yield


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
