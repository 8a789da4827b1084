"""The C-ABI library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments on the host before any device work."""
import ctypes as C
import os
import re

import pytest

from paper_2511_00855_amd import binding as B

HDR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "allanpoe.h")


def declared_symbols():
    text = open(HDR).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ap_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in allanpoe.h but not exported"


def test_struct_layouts_match_header_sizes():
    # field order/types of the ctypes mirrors follow the header; sizes are what a C compiler gives
    assert C.sizeof(B._Corpus) == 88
    assert C.sizeof(B._BuildParams) == 56
    assert C.sizeof(B._Queries) == 64
    assert C.sizeof(B._SearchParams) == 16


def test_host_side_argument_checks():
    lib = B.lib()
    h = C.c_void_p()
    bp = B.build_params(32)
    # NULL corpus
    assert lib.ap_build_index(None, C.byref(bp), None, C.byref(h)) == -1
    assert b"corpus" in lib.ap_last_error()
    cs = B._Corpus(100, 130, 0, 16, 16, 16, 16, 10, 16, 16, 16, 10)   # dim not a multiple of 4
    assert lib.ap_build_index(C.byref(cs), C.byref(bp), None, C.byref(h)) == -1
    assert b"dim" in lib.ap_last_error()
    cs = B._Corpus(100, 128, 7, 16, 16, 16, 16, 10, 16, 16, 16, 10)   # bad dtype
    assert lib.ap_ingest(C.byref(cs), C.byref(bp), None, C.byref(h)) == -1
    cs = B._Corpus(100, 128, 0, 16, 16, 16, 16, 10, 16, 16, 16, 10)
    bad = B.build_params(30)                                          # degree not a multiple of 4
    assert lib.ap_build_index(C.byref(cs), C.byref(bad), None, C.byref(h)) == -1
    assert b"degree" in lib.ap_last_error()
    bad = B.build_params(32, knn_k=16)
    assert lib.ap_build_index(C.byref(cs), C.byref(bad), None, C.byref(h)) == -1
    assert not h.value
    assert lib.ap_set_weights(None, (C.c_float * 3)(1, 1, 1)) == -1
    lib.ap_free_index(None)                                           # no-op


def test_debug_settings_are_named_and_bounded():
    lib = B.lib()
    for name in B.DEBUG_NAMES:
        B.debug_set(name, 0)
    assert lib.ap_debug_set(b"no_such_setting", C.c_int64(1)) == -1
    assert b"no_such_setting" in lib.ap_last_error()
    assert lib.ap_debug_set(b"seed_buffer_cap", C.c_int64(-5)) == -1
    assert lib.ap_debug_set(None, C.c_int64(0)) == -1
