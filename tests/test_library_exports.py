"""The C-ABI library loads and exports every entry point the header declares (no GPU work)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2601_00644_amd", "libflexverify.so")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "flexverify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fsv_[a-z_0-9]+)\s*\(", text)))


def _lib():
    if not os.path.exists(LIB):
        from paper_2601_00644_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ["fsv_create", "fsv_verify", "fsv_sample", "fsv_rollback", "fsv_destroy", "fsv_strerror"]:
        assert must in names


def test_every_declared_symbol_is_exported():
    lib = _lib()
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_names():
    from paper_2601_00644_amd import flexverify
    assert sorted(flexverify.EXPORTS) == declared_functions()


def test_strerror_and_null_arguments_fail_cleanly():
    lib = _lib()
    lib.fsv_strerror.restype = ctypes.c_char_p
    assert lib.fsv_strerror(0) == b"ok"
    assert b"invalid" in lib.fsv_strerror(-1)
    assert lib.fsv_create(None, None, None) == -1
    assert lib.fsv_verify(None, None, None, None) == -1
    lib.fsv_destroy(None)
