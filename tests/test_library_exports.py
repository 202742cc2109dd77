"""The C-ABI library loads and exports every symbol include/amap.h declares."""
import ctypes
import os
import re

from paper_2002_12798_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    hdr = open(os.path.join(ROOT, "include", "amap.h")).read()
    declared = set(re.findall(r"\b(amap_[a-z_]+)\s*\(", hdr))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)
