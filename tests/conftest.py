import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def _hip_runtime():
    """The HIP runtime this process has loaded (PyTorch's), for hipPeekAtLastError."""
    import ctypes
    try:
        with open("/proc/self/maps") as maps:
            for line in maps:
                if "libamdhip64" in line:
                    lib = ctypes.CDLL(line.split()[-1])
                    lib.hipPeekAtLastError.restype = ctypes.c_int
                    lib.hipGetLastError.restype = ctypes.c_int
                    return lib
    except OSError:
        pass
    return None


@pytest.fixture(autouse=True)
def no_error_left_in_the_runtime(request):
    """A library call must not leave an error behind in the HIP runtime: the caller's next,
    unrelated call (a PyTorch kernel launch) would report it as its own.  Checked after
    every GPU test, so that the test that leaves one is the test that fails."""
    yield
    if "gpu" not in request.keywords or not _have_gpu():
        return
    hip = _hip_runtime()
    if hip is None:
        return
    err = hip.hipPeekAtLastError()
    if err != 0:
        hip.hipGetLastError()      # taken back, so that the tests after this one start clean
        pytest.fail("the HIP runtime's last error is %d after this test" % err)
