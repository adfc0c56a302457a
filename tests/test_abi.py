"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed)."""
import ctypes
import os
import re

from paper_2511_11733_amd import dsd as D

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "dsd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dsd_[a-z_]+)\s*\(", src)))


def test_header_and_binding_agree():
    names = declared_functions()
    assert "dsd_stage_verify" in names and "dsd_accept" in names
    assert sorted(D.EXPORTS) == names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(D.LIB_PATH)
    for n in declared_functions():
        assert getattr(lib, n) is not None
    D.load()
    assert D.load().dsd_last_error() == b""


def test_struct_sizes_match_header_layout():
    assert ctypes.sizeof(D.ModelDesc) == 12 * 4
    assert ctypes.sizeof(D.AcceptParams) == 5 * 8 + 2 * 4 + 8 + 2 * 4
    assert ctypes.sizeof(D.AcceptStats) == 4 * 8
