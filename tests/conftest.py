import ctypes as C
import os
import subprocess
import sys

import numpy as np

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def orc():
    from oracle import oracle
    oracle.build_lib()
    return oracle


@pytest.fixture(scope="session")
def aten_philox(tmp_path_factory):
    """PyTorch's host Philox4x32-10 engine, compiled from its public header: an
    implementation of the published generator that this repository did not write."""
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    hdr = os.path.join(inc, "ATen", "core", "PhiloxRNGEngine.h")
    if not os.path.exists(hdr):
        pytest.skip("ATen Philox header not shipped with this torch build")
    so = str(tmp_path_factory.mktemp("aten") / "libaten_philox.so")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-I" + inc, "-o", so,
                           os.path.join(ROOT, "tests", "helpers", "aten_philox.cpp")])
    lib = C.CDLL(so)

    def f(seed, subsequence, offset):
        out = (C.c_uint32 * 4)()
        lib.aten_philox4x32_10(C.c_uint64(seed), C.c_uint64(subsequence), C.c_uint64(offset), out)
        return np.array(list(out), np.uint32)
    return f
