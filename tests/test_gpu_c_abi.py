"""The C ABI called from plain C++ (tests/c_abi_gpu_driver.cpp: hipMalloc'ed buffers, a stream
of its own, closed-form expected values), with no Python between the caller and the library:
the test only loads the small shared object and calls its one function."""
import ctypes
import os

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_caller_runs_clean():
    so = os.path.join(ROOT, "tests", "libc_abi_gpu_driver.so")
    assert os.path.exists(so), "tests/libc_abi_gpu_driver.so is not built: run __graft_entry__.build()"
    lib = ctypes.CDLL(so)
    lib.nz_c_abi_checks.restype = ctypes.c_int
    lib.nz_c_abi_checks.argtypes = []
    assert lib.nz_c_abi_checks() == 0, "a check in tests/c_abi_gpu_driver.cpp failed (its line is on stderr)"
