"""The C ABI library loads and exports every symbol that include/tbe355.h declares; argument checks that need
no GPU behave as documented.  No compute call is made here."""
import ctypes
import os
import re

import paper_2508_03854_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tbe355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tbe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = P.load_library()
    names = declared_symbols()
    assert len(names) >= 11
    for n in names:
        assert hasattr(L, n), n
    assert sorted(P.EXPORTS) == names


def test_status_strings_and_null_checks():
    L = P.load_library()
    assert L.tbe_status_string(0) == b"ok"
    assert all(L.tbe_status_string(i) for i in range(8))
    assert L.tbe_create(1, None, None, 0, None) == P.binding.EINVAL
    h = ctypes.c_void_p()
    rows = (ctypes.c_int64 * 1)(10)
    D = (ctypes.c_int32 * 1)(6)                       # not a multiple of 4
    assert L.tbe_create(1, rows, D, 0, ctypes.byref(h)) == P.binding.ESHAPE
    D = (ctypes.c_int32 * 1)(4)
    assert L.tbe_create(1, rows, D, 7, ctypes.byref(h)) == P.binding.EDTYPE
    assert L.tbe_create(0, rows, D, 0, ctypes.byref(h)) == P.binding.ESHAPE
    n = ctypes.c_size_t()
    assert L.tbe_workspace_bytes(None, 1, 1, ctypes.byref(n)) == P.binding.EINVAL
    assert L.tbe_destroy(None) == P.binding.OK
