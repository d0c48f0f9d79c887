"""CPU-only checks of the C ABI: the library loads and exports what include/recd.h declares, and
argument errors are reported as status codes before any GPU work."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2211_05239_amd", "librecd.so")


def _declared():
    text = open(os.path.join(ROOT, "include", "recd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(recd_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_calls():
    names = _declared()
    for n in ("recd_build_ikjt", "recd_pooled_lookup_unique", "recd_expand_inverse",
              "recd_backward_dedup", "recd_kjt_pooled_lookup", "recd_create", "recd_destroy"):
        assert n in names


@pytest.mark.skipif(not os.path.exists(LIB), reason="librecd.so not built (python -m paper_2211_05239_amd.build)")
def test_library_exports_every_declared_symbol():
    lib = C.CDLL(LIB)
    for n in _declared():
        assert hasattr(lib, n), n


@pytest.mark.skipif(not os.path.exists(LIB), reason="librecd.so not built")
def test_binding_lists_match_header():
    from paper_2211_05239_amd import recd
    assert sorted(recd.EXPORTED) == _declared()


@pytest.mark.skipif(not os.path.exists(LIB), reason="librecd.so not built")
def test_status_strings_and_null_context():
    lib = C.CDLL(LIB)
    lib.recd_status_string.restype = C.c_char_p
    assert lib.recd_status_string(0) == b"RECD_OK"
    assert lib.recd_status_string(-4) == b"RECD_EBOUNDS"
    lib.recd_last_error.restype = C.c_char_p
    lib.recd_last_error.argtypes = [C.c_void_p]
    assert lib.recd_last_error(None) == b"null context"
    lib.recd_set_option.argtypes = [C.c_void_p, C.c_int, C.c_int64]
    assert lib.recd_set_option(None, 1, 1) == -1
    assert lib.recd_destroy(None) == 0
    out = C.c_size_t(0)
    lib.recd_workspace_bytes.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int, C.POINTER(C.c_size_t)]
    assert lib.recd_workspace_bytes(64, 16384, 36_000_000, 128, C.byref(out)) == 0
    assert 0 < out.value < 8 << 30
    assert lib.recd_workspace_bytes(-1, 1, 1, 1, C.byref(out)) == -1


def test_product_has_no_oracle_import():
    """The product path must not reach into oracle/ (it would void every parity claim)."""
    pkg = os.path.join(ROOT, "paper_2211_05239_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text, fn
                assert "librecd_oracle" not in text, fn
