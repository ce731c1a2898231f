"""The C-ABI library loads without a GPU and exports every function include/bms.h declares."""
import ctypes
import os
import re

from paper_2311_02909_amd import bms

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "bms.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bms_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary_calls():
    names = _declared_functions()
    for required in ("bms_csr_load", "bms_sample_nodewise", "bms_sample_ladies", "bms_free"):
        assert required in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(bms.LIB_PATH)
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_error_strings_and_argument_checks_need_no_gpu():
    lib = bms.lib()
    assert lib.bms_strerror(0) == b"success"
    assert b"invalid" in lib.bms_strerror(bms.EINVAL)
    out = ctypes.c_void_p()
    # null rowptr is rejected before any device call
    rc = lib.bms_csr_load(None, None, 4, 0, bms.HOST, ctypes.byref(out))
    assert rc == bms.EINVAL and not out.value
    assert b"null" in lib.bms_last_error()
    # a handle that is not a csr
    junk = (ctypes.c_uint32 * 4)(0, 0, 0, 0)
    fan = (ctypes.c_int32 * 1)(5)
    seeds = (ctypes.c_int32 * 2)(0, 1)
    rc = lib.bms_sample_nodewise(ctypes.addressof(junk), seeds, 1, 2, fan, 1, 0, None, ctypes.byref(out))
    assert rc == bms.EINVAL and not out.value
    lib.bms_free(None)
