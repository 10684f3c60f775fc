"""The C-ABI library loads and exports every entry point include/akvq.h declares; host-only helpers behave.
No kernel is launched here (runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2501_15021_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2501_15021_amd import build
        build.build()
    return binding.lib()


def test_every_declared_symbol_is_exported(L):
    from paper_2501_15021_amd import binding
    header = open(os.path.join(ROOT, "include", "akvq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(akvq_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_host_helpers(L):
    from paper_2501_15021_amd.binding import akvq_cache
    assert L.akvq_version() >= 100
    assert L.akvq_strerror(0) == b"ok" and L.akvq_strerror(-3) == b"capacity exceeded"
    sizes = (C.c_size_t * 8)()
    shape = akvq_cache(2, 4, 128, 128, 64, 0)
    assert L.akvq_cache_bytes(C.byref(shape), sizes) == 0
    bh = 8
    assert list(sizes) == [bh * 4 * 1024, bh * 4 * 1024, bh * 128 * 4, bh * 128 * 4, bh * 64 * 256, bh * 64 * 256,
                           bh * 64 * 4, 32]
    shape64 = akvq_cache(2, 4, 64, 128, 64, 0)
    assert L.akvq_cache_bytes(C.byref(shape64), sizes) == 0 and sizes[2] == bh * 128 * 8
    for bad, code in ((akvq_cache(2, 4, 32, 128, 64, 0), -2), (akvq_cache(2, 4, 128, 100, 64, 0), -1),
                      (akvq_cache(0, 4, 128, 128, 64, 0), -1), (akvq_cache(2, 4, 128, 128, 64, 129), -3)):
        assert L.akvq_cache_bytes(C.byref(bad), sizes) == code
    assert L.akvq_decode_workspace_bytes(2, 8, 4) >= 2 * 8 * 4 * 132 * 4
    assert L.akvq_decode_workspace_bytes(0, 8, 4) == 0
    assert L.akvq_select_workspace_bytes(1, 32, 32, 640, 64) >= 32 * 1 * 64 * 2 * 4 + 32 * 640 * 4  # row statistics + masses
    for args in ((1, 32, 640), (16, 32, 4096), (64, 32, 8192), (32, 4, 32768), (1, 1, 1)):
        n = L.akvq_decode_default_splits(*args)
        assert 1 <= n <= 64 and n <= max(1, (args[2] + 63) // 64)


def test_argument_errors_launch_nothing(L):
    """Null pointers are rejected on the host before any launch (safe without a GPU)."""
    from paper_2501_15021_amd.binding import akvq_cache
    c = akvq_cache(1, 1, 128, 64, 64, 0)  # all device pointers null
    assert L.akvq_quantize_append(C.byref(c), None, None, 1, 0.8, 0, None) == -1
    assert L.akvq_decode_attention(C.byref(c), None, 1, 0.1, None, None, 1, None, 0, 0, None) == -1
    assert L.akvq_select_salient(C.byref(c), 0, None, None, 1, None, 64, 0, 0, 0.0, None, None, 0, None) == -1
