"""CPU-side checks of the C boundary: the built library exports every function the header
declares, and the calls that need no GPU validate their arguments."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2508_06041_amd", "libdpllm.so")
HEADER = os.path.join(ROOT, "include", "dpllm.h")


def declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dpllm_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    return C.CDLL(LIB)


def test_header_declares_the_four_calls_of_the_path():
    names = declared()
    for need in ("dpllm_load_linear", "dpllm_estimate", "dpllm_gemv", "dpllm_decode_step"):
        assert need in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_names():
    import importlib.util
    spec = importlib.util.spec_from_file_location("b", os.path.join(ROOT, "paper_2508_06041_amd", "binding.py"))
    src = open(spec.origin).read()
    listed = set(re.findall(r'"(dpllm_[a-z_]+)"', src))
    assert set(declared()) <= listed


def test_device_bytes_validates_without_a_gpu(lib):
    n = C.c_size_t(0)
    f = lib.dpllm_linear_device_bytes
    f.argtypes = [C.c_int] * 4 + [C.POINTER(C.c_size_t)]
    assert f(1024, 1024, 4, 3, C.byref(n)) == 0
    planes = 4 * 1024 * 1024 // 8
    luts = 1024 * (8 + 16) * 2
    assert n.value >= planes + luts and n.value % 256 == 0
    assert f(1024, 1000, 4, 3, C.byref(n)) == -2      # in % 32 != 0
    assert f(0, 1024, 4, 3, C.byref(n)) == -2
    assert f(8, 32, 9, 3, C.byref(n)) == -3           # p > 8
    assert f(8, 32, 4, 5, C.byref(n)) == -3           # kmin > p
    assert f(8, 32, 4, 3, None) == -1
