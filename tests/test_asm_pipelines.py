"""The hand-counted load pipelines of the HIP kernels, checked on the compiler's own output (CPU only:
hipcc cross-compiles to a listing).  The tiled GEMM keeps weight fragments in flight in registers that
inline asm loads into, with `s_waitcnt vmcnt(N)` counted by hand; nothing in the language stops the
compiler from moving or spilling such a register early, so every build is checked: along every path
of every kernel, no instruction may touch a register whose load the wait counts say is still
outstanding.  The checker itself is pinned on two tiny listings, one clean and one with the hazard."""
import os
import subprocess
import tempfile

import pytest

from tests import asm_pending as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_11733_amd", "csrc")

CLEAN = """
k_clean:
	global_load_dwordx4 v[4:7], v[0:1], off
	global_load_dwordx4 v[8:11], v[0:1], off
	v_add_u32_e32 v2, 1, v2
	s_waitcnt vmcnt(1)
	v_add_f32_e32 v3, v4, v5
	s_waitcnt vmcnt(0)
	v_add_f32_e32 v3, v8, v9
	s_endpgm
"""
HAZARD = """
k_hazard:
	global_load_dwordx4 v[4:7], v[0:1], off
	global_load_dwordx4 v[8:11], v[0:1], off
	s_waitcnt vmcnt(1)
	v_add_f32_e32 v3, v8, v9
	s_endpgm
k_hazard_on_one_branch:
	global_load_dwordx4 v[4:7], v[0:1], off
	s_cbranch_scc1 .LBB1_2
	s_waitcnt vmcnt(0)
.LBB1_2:
	v_mov_b32_e32 v12, v5
	s_endpgm
"""


def violations(text):
    with tempfile.NamedTemporaryFile("w", suffix=".s", delete=False) as f:
        f.write(text)
        path = f.name
    try:
        return {name: A.check_kernel(path, name, k) for name, k in A.parse(path).items()}
    finally:
        os.unlink(path)


def test_checker_flags_a_register_touched_while_its_load_is_in_flight():
    assert violations(CLEAN) == {"k_clean": 0}
    got = violations(HAZARD)
    assert got["k_hazard"] == 1 and got["k_hazard_on_one_branch"] == 1


@pytest.mark.parametrize("src", ["dsd_gemm_tiled.hip", "dsd_stage_bf16.hip"])
def test_no_kernel_touches_a_register_with_a_load_in_flight(src, tmp_path):
    from paper_2511_11733_amd import build as B

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = str(tmp_path / (src + ".s"))
    flags = [f for f in B.FLAGS if f != "-fPIC"]
    r = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", out],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    kernels = A.parse(out)
    assert len(kernels) >= 5
    bad = {name: n for name, k in kernels.items() if (n := A.check_kernel(out, name, k))}
    assert not bad, f"{src}: instructions touch registers with loads in flight: {bad}"
