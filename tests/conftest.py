import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def aten_philox(tmp_path_factory):
    """Third-party Philox4x32-10 (the header-only engine that ships with PyTorch),
    compiled for the host; the pin for the oracle's own Philox."""
    import ctypes
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "aten_philox_shim.cpp")
    out = str(tmp_path_factory.mktemp("aten") / "libaten_philox_shim.so")
    subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-I", inc, src, "-o", out],
                   check=True)
    lib = ctypes.CDLL(out)
    lib.aten_philox_block.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                      ctypes.c_void_p]
    lib.aten_philox_block.restype = None

    def block(seed, subsequence, offset):
        import numpy as np
        o = np.zeros(4, dtype=np.uint32)
        lib.aten_philox_block(seed, subsequence, offset, o.ctypes.data_as(ctypes.c_void_p))
        return o

    return block
