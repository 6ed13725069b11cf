"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

from paper_2511_15898_amd.binding import EXPORTS
from paper_2511_15898_amd.build import LIB_PATH, ROOT, build_library


def _declared():
    text = open(os.path.join(ROOT, "include", "gr_verify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gr_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared() == sorted(EXPORTS)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB_PATH):
        build_library()
    lib = ctypes.CDLL(LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    lib.gr_strerror.restype = ctypes.c_char_p
    assert lib.gr_strerror(0) == b"ok" and b"support" in lib.gr_strerror(-5)
