"""The C-ABI library loads and exports every entry point the header declares
(no GPU needed: nothing is called)."""
import ctypes
import os
import re

from paper_2410_09687_amd import moin

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moin.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moin_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared() == sorted(moin.EXPORTS)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(moin.LIB_PATH):
        from paper_2410_09687_amd.build import build_libmoin
        build_libmoin()
    lib = ctypes.CDLL(moin.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    moin.load()
    assert moin._strerror(0) == "success"
    assert "invalid" in moin._strerror(-1)
