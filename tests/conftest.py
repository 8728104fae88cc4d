import ctypes
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def rocrand_pin():
    """rocRAND's host-callable Threefry-2x32-20 engine behind a C function (test-only library)."""
    src = os.path.join(ROOT, "tests", "pins", "rocrand_threefry_pin.cpp")
    out = os.path.join(ROOT, "tests", "pins", "librocrand_pin.so")
    if not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        hipcc = "/opt/rocm/bin/hipcc"
        if not os.path.exists(hipcc):
            pytest.skip("hipcc not available to build the rocRAND pin")
        subprocess.check_call([hipcc, "-x", "hip", "--cuda-host-only", "-O1", "-fPIC", "-shared",
                               "-o", out, src], stderr=subprocess.DEVNULL)
    lib = ctypes.CDLL(out)

    def words(seed, subsequence, offset, n):
        buf = np.empty(n, np.uint32)
        lib.pin_rocrand_threefry2x32_20(ctypes.c_ulonglong(seed), ctypes.c_ulonglong(subsequence),
                                        ctypes.c_ulonglong(offset), ctypes.c_int(n),
                                        buf.ctypes.data_as(ctypes.c_void_p))
        return buf

    def block(counter, key):
        """Threefry(key=(k0,k1), counter=(c0,c1)) through rocRAND: seed = k1:k0, offset = 2*c0,
        subsequence = c1."""
        seed = (int(key[1]) << 32) | int(key[0])
        return words(seed, int(counter[1]), 2 * int(counter[0]), 2)

    return type("Pin", (), {"words": staticmethod(words), "block": staticmethod(block)})
