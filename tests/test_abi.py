"""The C-ABI library builds for gfx950, loads without a GPU and exports every
function that include/tbe.h declares.  No compute call is made here."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tbe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tbe_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2305_01515_amd import tbe
    lib = tbe.lib()
    names = declared_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in tbe.h but not exported"
    assert sorted(tbe.EXPORTS) == names


def test_library_holds_gfx950_code():
    from paper_2305_01515_amd import tbe
    tbe.lib()
    blob = open(tbe.LIB_PATH, "rb").read()
    assert b"gfx950" in blob


def test_host_side_argument_checks_need_no_gpu():
    from paper_2305_01515_amd import tbe
    lib = tbe.lib()
    h = ctypes.c_void_p()
    assert lib.tbe_create(ctypes.byref(h), None, 0, 32, 1, 1, None, None) == -1
    assert lib.tbe_create(None, None, 1, 32, 1, 1, None, None) == -1
    assert b"" != lib.tbe_last_error(None)
    assert lib.tbe_prefetch(None, None, None, 1, 1) == -1
    assert lib.tbe_flush(None) == -1
