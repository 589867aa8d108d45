"""The C-ABI library loads and exports every entry point the header declares.
No compute call is made here (no GPU needed)."""
from __future__ import annotations

import ctypes as C
import os
import re

import pytest

from paper_2501_08547_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "omega_srpe.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(omg_[a-z_]+)\s*\(", text)))


def test_library_is_built():
    assert os.path.exists(B.LIB_PATH), "run `python -m paper_2501_08547_amd.build` first"


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert len(names) >= 14
    L = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(L, n), f"{n} is declared in the header but not exported"
    assert sorted(B.EXPORTS) == names


def test_every_export_has_argument_types_that_match_the_header():
    """A function without declared argument types gets Python ints as 32-bit C ints: a device address
    would arrive truncated.  The number of declared types must equal the header's parameter count."""
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    L = B.lib()
    for name in B.EXPORTS:
        m = re.search(r"\b%s\s*\(([^;]*?)\)\s*;" % name, text, flags=re.S)
        assert m, name
        params = m.group(1).strip()
        n_params = 0 if params in ("", "void") else params.count(",") + 1
        fn = getattr(L, name)
        assert fn.argtypes is not None, f"{name}: no argument types in binding.py"
        assert len(fn.argtypes) == n_params, f"{name}: {len(fn.argtypes)} types for {n_params} parameters"


def test_binding_structs_match_header_layout():
    assert C.sizeof(B.omg_base_csr) == 24
    assert C.sizeof(B.omg_table) == 32
    assert C.sizeof(B.omg_layer) == 32 + 6 * 8 + 8 + 8 + 16 + 8  # 8 four-byte fields, 6 pointers, 2 floats, float + pad, pointer, int64, pointer
    assert C.sizeof(B.omg_timing) == 4 * (2 + 3 * B.OMG_MAX_LAYERS)


def test_error_strings_and_host_side_argument_checks():
    L = B.lib()
    assert L.omg_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -6):
        assert len(L.omg_strerror(code)) > 0
    handle = C.c_void_p(None)
    assert L.omg_create(C.byref(handle), None, None) == B.OMG_EINVAL
    bad = B.omg_base_csr(0, None, None)
    assert L.omg_create(C.byref(handle), C.byref(bad), None) == B.OMG_EINVAL
    assert not handle
    sizes = (C.c_int64 * 4)()
    assert L.omg_graph_sizes(None, C.byref(sizes)) == B.OMG_EINVAL
    assert L.omg_set_profiling(None, 1) == B.OMG_EINVAL
    assert L.omg_last_graph_sizes(None, C.byref(sizes)) == B.OMG_ESTATE
    nbytes, ms = C.c_double(0.0), C.c_float(0.0)
    assert L.omg_measure_read_rate(None, None, 1 << 20, 1, 1, C.byref(nbytes), C.byref(ms)) == B.OMG_EINVAL
