"""The C-ABI library loads and exports every symbol include/pvf.h declares (no GPU needed)."""
import ctypes
import os
import re

from paper_2601_12247_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pvf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pvf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layouts_match_header_sizes():
    assert ctypes.sizeof(B.ModelCfgC) == 9 * 4
    assert ctypes.sizeof(B.DecodeCfgC) == 13 * 4
    assert ctypes.sizeof(B.StateC) == 19 * 8
    assert ctypes.sizeof(B.WeightsC) == 9 * 8
    assert ctypes.sizeof(B.StatsC) == 2 * 4 + 5 * 8 + 8


def test_argument_errors_are_reported_without_a_gpu():
    L = B.lib()
    # NULL pointers are rejected before any launch
    assert L.pvf_stage1(None, None, 0, 1, 16, 0, 1.0, None, None) == -1
    assert b"NULL" in L.pvf_last_error(None)
    assert L.pvf_gemm(None, 7, None, None, None, None, 1, 1, 1) == -1
    h = ctypes.c_void_p()
    assert L.pvf_create(ctypes.byref(h), None, None, 1, 1, 1) == -1
    assert L.pvf_forward(None, None, None, 1, 1, None, 1, None) == -1
