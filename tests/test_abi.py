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


def test_bf16_values_convert_to_fp16_without_loss_in_the_stated_range():
    """The matrix-core path stores bf16 projection weights as fp16 and calls that exact for magnitudes
    2^-17 .. 65504; smaller ones may move by at most half of fp16's subnormal spacing (2^-25).  Checked
    over every bf16 bit pattern."""
    import numpy as np
    bits = np.arange(1 << 16, dtype=np.uint32)
    v = (bits << 16).view(np.float32)
    fin = np.isfinite(v)
    mag = np.abs(v)
    with np.errstate(over="ignore"):
        back = v.astype(np.float16).astype(np.float32)
    exact = fin & ((mag == 0) | ((mag >= 2.0 ** -17) & (mag <= 65504.0)))
    assert exact.sum() == 33 * 128 * 2 + 2          # exponents -17 .. 15, both signs, and the two zeros
    np.testing.assert_array_equal(back[exact], v[exact])
    small = fin & (mag < 2.0 ** -17)
    assert np.abs(back[small].astype(np.float64) - v[small].astype(np.float64)).max() <= 2.0 ** -25
