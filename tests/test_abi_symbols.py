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


@pytest.mark.parametrize("out,in_,p", [(1, 32, 3), (70, 160, 4), (64, 128, 8), (130, 288, 6)])
def test_device_layout_is_a_permutation_with_the_stated_structure(lib, out, in_, p):
    """The private layout of the planes, computed on the host (no GPU): every (plane, row, column) bit has a
    place of its own inside its plane's region; the four 32-column words of a row inside a 128-column tile are
    16 contiguous bytes and the 64 rows of a tile 1 KiB (what a lane and a wavefront load at once); the bits of one
    weight sit in the same word index of every plane at positions that descend by one from plane to plane (what
    lets a k-bit code be assembled by merging whole words under masks, for every k); columns 2i and 2i+1 sit
    three positions apart in plane 0 (the two fields of one byte of the merged words at k = 3)."""
    f = lib.dpllm_debug_locate
    f.argtypes = [C.c_int] * 7 + [C.POINTER(C.c_size_t), C.POINTER(C.c_int)]
    n = C.c_size_t(0)
    g = lib.dpllm_linear_device_bytes
    g.argtypes = [C.c_int] * 4 + [C.POINTER(C.c_size_t)]
    assert g(out, in_, p, 3, C.byref(n)) == 0
    nrq, ncc = (out + 63) // 64, (in_ // 32 + 3) // 4
    plane_bytes = nrq * ncc * 1024
    assert n.value >= p * plane_bytes

    def where(plane, row, col):
        off, bit = C.c_size_t(0), C.c_int(0)
        assert f(out, in_, p, 3, plane, row, col, C.byref(off), C.byref(bit)) == 0
        return off.value, bit.value

    seen = set()
    for plane in range(p):
        for row in range(out):
            for col in range(in_):
                off, bit = where(plane, row, col)
                assert off % 4 == 0 and 0 <= bit < 32
                assert plane * plane_bytes <= off < (plane + 1) * plane_bytes, (plane, row, col)
                assert (off, bit) not in seen
                seen.add((off, bit))
    for row in (0, out - 1):
        for col in range(0, in_, 32):
            off0, bit0 = where(0, row, col)
            # tile structure: word (col / 32) % 4 of the row's 16 bytes; rows of a tile 16 bytes apart
            tile = (row // 64) * ncc + col // 128
            assert off0 == tile * 1024 + (row % 64) * 16 + (col // 32 % 4) * 4
            for c in range(col, col + 32):
                o0, b0 = where(0, row, c)
                assert o0 == off0
                for plane in range(1, p):
                    o, b = where(plane, row, c)
                    assert o - plane * plane_bytes == o0 and b == (b0 - plane) % 32
            for c in range(col, col + 32, 2):
                assert (where(0, row, c)[1] - where(0, row, c + 1)[1]) % 32 == 3
    off, bit = C.c_size_t(0), C.c_int(0)
    assert f(out, in_, p, 3, p, 0, 0, C.byref(off), C.byref(bit)) == -3       # plane out of range
    assert f(out, in_, p, 3, 0, out, 0, C.byref(off), C.byref(bit)) == -3
    assert f(out, in_, p, 3, 0, 0, in_, C.byref(off), C.byref(bit)) == -3
    assert f(out, in_, p, 3, 0, 0, 0, None, C.byref(bit)) == -1


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits with an error before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
