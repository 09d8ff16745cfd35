"""CPU-side checks of the boundary: the built library loads and exports every symbol that
include/stand.h declares (no compute calls are made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2506_04708_amd", "libstand.so")
HEADER = os.path.join(ROOT, "include", "stand.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(stand_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_named_calls():
    names = _declared()
    for n in ("stand_update", "stand_draft", "stand_verify", "stand_step"):
        assert n in names


@pytest.mark.skipif(not os.path.exists(LIB), reason="libstand.so not built (run __graft_entry__.build())")
def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    for n in _declared():
        assert hasattr(lib, n), n
    lib.stand_strerror.restype = ctypes.c_char_p
    assert lib.stand_strerror(0) == b"ok" and b"invalid" in lib.stand_strerror(-1)


@pytest.mark.skipif(not os.path.exists(LIB), reason="libstand.so not built")
def test_binding_lists_the_same_symbols():
    from paper_2506_04708_amd import binding
    assert sorted(binding.EXPORTED) == _declared()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_04708_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "stand_oracle" not in src and "from oracle" not in src, f
