"""The C-ABI library loads without a GPU and exports every function include/bms.h declares."""
import ctypes
import os
import re

import pytest

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


def test_header_compiles_as_c_and_cpp_and_structs_match_the_binding(tmp_path):
    # the binding mirrors three structs of the header with ctypes: sizes and field offsets must agree
    import subprocess
    src = tmp_path / "layout.c"
    fields = {
        "bms_opts": [f[0] for f in bms._Opts._fields_],
        "bms_hop_view": [f[0] for f in bms._HopView._fields_],
        "bms_mb_view": [f[0] for f in bms._MbView._fields_],
    }
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "bms.h"', "int main(void) {"]
    for struct, names in fields.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (struct, struct))
        for n in names:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (struct, n, struct, n))
    lines += ["return 0; }"]
    src.write_text("\n".join(lines))
    inc = os.path.join(ROOT, "include")
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", inc, "-o", str(exe), str(src)])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc,
                           os.path.join(inc, "bms.h")])
    got = dict(line.split() for line in subprocess.check_output([str(exe)], text=True).splitlines())
    mirrors = {"bms_opts": bms._Opts, "bms_hop_view": bms._HopView, "bms_mb_view": bms._MbView}
    for struct, cls in mirrors.items():
        assert int(got[struct]) == ctypes.sizeof(cls), struct
        for n in fields[struct]:
            assert int(got["%s.%s" % (struct, n)]) == getattr(cls, n).offset, (struct, n)
    # and the flag values the binding hard-codes are the header's
    text = open(os.path.join(inc, "bms.h")).read()
    for name in ("LADIES_SQUARED", "PROFILE", "EXTRACT_BUCKETS", "EXTRACT_BITMAP", "EXTRACT_SORT", "LADIES_DENSE",
                 "PROFILE_MAIN", "UNION_DST", "NODEWISE_REPLACE", "ASYNC", "LADIES_NO_INDEX"):
        m = re.search(r"#define\s+BMS_%s\s+(\d+)u" % name, text)
        assert m and int(m.group(1)) == getattr(bms, name), name


def test_probe_library_exports_its_two_entry_points():
    # the rate probes behind `bench.py --line-probe / --lds-probe` live in a library of their own
    import ctypes
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2311_02909_amd", "libbms_probe.so")
    if not os.path.exists(path):
        pytest.skip("libbms_probe.so is not built (python paper_2311_02909_amd/build.py)")
    P = ctypes.CDLL(path)
    for name in ("bms_probe_random_rows", "bms_probe_lds_ops"):
        assert hasattr(P, name), name
    # arguments are checked before anything is launched
    P.bms_probe_random_rows.restype = ctypes.c_int
    assert P.bms_probe_random_rows(None, 0, None, 0, 3, 0, None, None) == -1
    assert P.bms_probe_lds_ops(None, 0, 0, 5, 0, None) == -1
