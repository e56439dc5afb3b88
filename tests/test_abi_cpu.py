"""No-GPU checks of the boundary: the shared library loads and exports every
entry point the header declares; the binding's name list matches the header."""
import ctypes
import os
import re

from paper_2509_09424_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ensi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ensi_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared() == sorted(binding.EXPORTED)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name


def test_error_codes_and_null_handling_without_gpu():
    lib = binding.load()
    # argument validation happens before any device call
    assert lib.ensi_ctx_create(None, None) == -1
    assert lib.ensi_last_error(None) == b"null context"
    bad = binding._Params(3, 50, 2, 60, 1, 1, 40, 0)  # log_n below the supported range
    h = ctypes.c_void_p()
    assert lib.ensi_ctx_create(ctypes.byref(bad), ctypes.byref(h)) == -1 and not h.value
