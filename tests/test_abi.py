"""Host-side checks of the C ABI: the library loads, exports every symbol that
include/solar.h declares, and rejects bad arguments without touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "solar.h")
LIB = os.path.join(ROOT, "paper_2603_02561_amd", "libsolar.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(solar_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2603_02561_amd import build
        build.build_library()
    return ctypes.CDLL(LIB)


def test_header_declares_the_entry_points():
    names = declared_functions()
    for must in ("solar_svd_factorize", "solar_svd_attention", "solar_dense_attention_ref",
                 "solar_gram", "solar_workspace_bytes", "solar_status_string"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in solar.h but not exported"


def test_status_strings_and_workspace_size(lib):
    lib.solar_status_string.restype = ctypes.c_char_p
    lib.solar_status_string.argtypes = [ctypes.c_int]
    seen = {lib.solar_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and "ok" in seen and "unknown status" not in seen
    assert lib.solar_status_string(99).decode() == "unknown status"
    lib.solar_workspace_bytes.restype = ctypes.c_size_t
    lib.solar_workspace_bytes.argtypes = [ctypes.c_int] * 6
    small = lib.solar_workspace_bytes(1, 1024, 64, 8, 64, 0)
    big = lib.solar_workspace_bytes(64, 10000, 128, 32, 1000, 1)
    assert 0 < small < big and big % 256 == 0
    assert lib.solar_workspace_bytes(1, 1024, 100, 8, 64, 0) == 0     # unsupported d


def test_argument_validation_happens_before_any_launch(lib):
    """Null pointers, bad sizes and unsupported shapes return a status code on the host;
    no device pointer is dereferenced and no kernel is launched (there is no GPU here)."""
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.solar_svd_factorize.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.solar_svd_factorize.restype = ci
    fake = 0x1000  # never dereferenced: every call below must fail validation first
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    assert lib.solar_svd_factorize(None, None, 1, 64, 64, 8, 0, fake, fake, None, None, fake, 1 << 30, None) == INVALID
    assert lib.solar_svd_factorize(fake, None, 0, 64, 64, 8, 0, fake, fake, None, None, fake, 1 << 30, None) == INVALID
    assert lib.solar_svd_factorize(fake, None, 1, 64, 64, 65, 0, fake, fake, None, None, fake, 1 << 30, None) == INVALID
    assert lib.solar_svd_factorize(fake, None, 1, 4, 64, 8, 0, fake, fake, None, None, fake, 1 << 30, None) == INVALID
    assert lib.solar_svd_factorize(fake, None, 1, 64, 64, 8, 7, fake, fake, None, None, fake, 1 << 30, None) == INVALID
    assert lib.solar_svd_factorize(fake, None, 1, 640, 96, 8, 0, fake, fake, None, None, fake, 1 << 30, None) == UNSUPPORTED
    assert lib.solar_svd_factorize(fake, None, 1, 640, 256, 48, 0, fake, fake, None, None, fake, 1 << 30, None) == UNSUPPORTED
    assert lib.solar_svd_factorize(fake, None, 1, 640, 64, 8, 0, fake, fake, None, None, None, 0, None) == WORKSPACE
    assert lib.solar_svd_factorize(fake, None, 1, 640, 64, 8, 0, fake, fake, None, None, fake, 16, None) == WORKSPACE
    assert lib.solar_svd_factorize(fake, None, 1, 640, 64, 8, 0, fake, fake, None, None, 0x1010, 1 << 30, None) == WORKSPACE
    # the allocation-free variant: same checks, and sizes beyond its built-in scratch array
    lib.solar_svd_factorize_static.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp]
    lib.solar_svd_factorize_static.restype = ci
    SCRATCH_LIMIT = 6
    assert lib.solar_svd_factorize_static(None, None, 1, 64, 64, 8, 0, fake, fake, None, None, None) == INVALID
    assert lib.solar_svd_factorize_static(fake, None, 1, 640, 96, 8, 0, fake, fake, None, None, None) == UNSUPPORTED
    assert lib.solar_svd_factorize_static(fake, None, 64, 100000, 256, 32, 1, fake, fake, None, None, None) == SCRATCH_LIMIT
    lib.solar_svd_attention.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, cf, ci, ci, vp, vp, sz, vp]
    lib.solar_svd_attention.restype = ci
    assert lib.solar_svd_attention(fake, fake, fake, None, None, 1, 64, 64, 8, 4, 1.0, 0, 0, fake, None, 0, None) == INVALID
    assert lib.solar_svd_attention(fake, None, fake, None, None, 1, 64, 64, 8, 4, 1.0, 1, 0, fake, None, 0, None) == INVALID
    assert lib.solar_svd_attention(fake, fake, fake, fake, None, 1, 64, 64, 8, 4, 1.0, 9, 0, fake, None, 0, None) == INVALID
    assert lib.solar_svd_attention(fake, fake, fake, fake, None, 1, 64, 64, 8, 0, 1.0, 0, 0, fake, None, 0, None) == INVALID
    lib.solar_dense_attention_ref.argtypes = [vp, vp, vp, ci, ci, ci, ci, cf, ci, vp, vp, sz, vp]
    lib.solar_dense_attention_ref.restype = ci
    assert lib.solar_dense_attention_ref(fake, None, None, 1, 64, 64, 4, 1.0, 0, fake, None, 0, None) == INVALID
    assert lib.solar_dense_attention_ref(fake, fake, None, 1, 64, 512, 4, 1.0, 0, fake, None, 0, None) == UNSUPPORTED
    lib.solar_gram.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, sz, vp]
    lib.solar_gram.restype = ci
    assert lib.solar_gram(fake, None, 1, 64, 64, 0, None, fake, 1 << 30, None) == INVALID
    assert lib.solar_gram(fake, None, 1, 64, 48, 0, fake, fake, 1 << 30, None) == UNSUPPORTED


def test_info_status_and_debug_options(lib):
    """Host-side helpers: the verdict over a per-user info array (host memory) and the debug
    switches, which only store a value."""
    lib.solar_info_status.argtypes = [ctypes.c_void_p, ctypes.c_int]
    lib.solar_info_status.restype = ctypes.c_int
    OK, INVALID, NOT_CONVERGED = 0, 1, 5

    def verdict(values):
        arr = (ctypes.c_int32 * len(values))(*values)
        return lib.solar_info_status(arr, len(values))
    assert verdict([0, 0, 0]) == OK
    assert verdict([0, 7, 0]) == NOT_CONVERGED
    assert verdict([0, 7, -1]) == INVALID
    assert lib.solar_info_status(None, 3) == INVALID
    lib.solar_debug_option.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.solar_debug_option.restype = ctypes.c_int
    assert lib.solar_debug_option(0, 3) == OK and lib.solar_debug_option(0, 0) == OK
    assert lib.solar_debug_option(0, -1) == INVALID
    assert lib.solar_debug_option(1, 1) == OK and lib.solar_debug_option(1, 0) == OK
    assert lib.solar_debug_option(9, 1) == INVALID
