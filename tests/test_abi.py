"""Host-only checks of the C ABI: the library loads and exports every symbol include/jz.h declares, and
argument validation that needs no GPU returns the documented codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def jzlib():
    from paper_1807_11205_amd import api
    if not os.path.exists(api.LIB_PATH):
        from paper_1807_11205_amd import build
        build.build()
    return api


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "jz.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(jz_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(jzlib):
    L = jzlib.lib()
    names = declared_symbols()
    assert len(names) >= 11
    for n in names:
        assert hasattr(L, n), n
    assert sorted(jzlib.EXPORTS) == names


def test_status_strings_and_version(jzlib):
    assert jzlib.jz_version() >= 100
    assert jzlib.status_string(0) == "JZ_OK"
    for code in range(-8, 0):
        assert jzlib.status_string(code).startswith("JZ_ERR_")
    assert "unknown" in jzlib.status_string(-99)


def test_lars_table_validation_on_the_host(jzlib):
    import numpy as np
    L = jzlib.lib()
    n = ctypes.c_size_t(0)

    def ps(offsets, flags):
        o = np.asarray(offsets, np.int64)
        f = np.asarray(flags, np.uint8)
        s = jzlib.jz_param_set(len(flags), o.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                               f.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), None, None, None, None)
        s._keep = (o, f)
        return s

    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 64, 4160], [3, 2])), ctypes.byref(n)) == 0 and n.value > 0
    small = n.value
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 64, 4160000], [3, 2])), ctypes.byref(n)) == 0 and n.value > small
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0], [])), ctypes.byref(n)) == 0
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([8, 64], [3])), ctypes.byref(n)) == jzlib.JZ_ERR_SHAPE       # offsets[0] != 0
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 64, 32], [3, 3])), ctypes.byref(n)) == jzlib.JZ_ERR_SHAPE  # decreasing
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 2 ** 31], [3])), ctypes.byref(n)) == jzlib.JZ_ERR_UNSUPPORTED
    assert L.jz_lars_workspace_bytes(None, ctypes.byref(n)) == jzlib.JZ_ERR_NULL
    assert L.jz_lars_workspace_bytes(ctypes.byref(ps([0, 8], [3])), None) == jzlib.JZ_ERR_NULL
