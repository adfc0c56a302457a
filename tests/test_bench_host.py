"""Host logic of bench.py (no GPU): the byte accounting behind the roofline figures, the parser of the
committed counter summaries, the thresholds it feeds the accept step, and the one-GPU rule."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2511_11733_amd import workloads as W  # noqa: E402


def test_algorithmic_bytes_counts_every_weight_and_cached_element_once():
    """c2 by hand: 8 layers of an 8B-shaped block in bf16, the K/V of one sequence of 2048 positions, the
    appended rows and the hidden rows in and out."""
    cfg = W.CONFIGS["c2"]
    m = cfg.model
    qd, kd = m.Hq * m.hd, m.Hkv * m.hd
    per_layer = (m.d * (qd + 2 * kd) + qd * m.d + 3 * m.F * m.d + 2 * m.d) * 2
    kv = 2 * cfg.B * m.Hkv * cfg.C * m.hd * 2
    rows = cfg.B * cfg.k
    expected = m.L * (per_layer + kv + 2 * rows * kd * 2) + 2 * rows * m.d * 2
    got = bench.algorithmic_bytes(cfg)
    total = got["total"] if isinstance(got, dict) else got[0] if isinstance(got, tuple) else got
    assert abs(total - expected) <= 1e-3 * expected, (total, expected)


def test_traffic_is_read_from_the_counter_table_not_the_timing_table():
    """Every committed summary lists the dominant kernel twice (timings, then counters); the bytes must be
    the counter line's read + written MB, which for a weight-streaming GEMM is about its algorithmic bytes."""
    for name, match, lo, hi in (("c4", "gemm_tiled_kernel<3, 7, 1>", 0.93e9, 1.0e9),
                                ("c3", "gemm_tiled_kernel<8, 4, 1>", 0.23e9, 0.27e9)):
        traffic, src = bench.committed_traffic(name, match)
        assert src == f"profiles/verify_step_{name}.txt"
        assert lo < traffic < hi, (name, traffic)
    assert bench.committed_traffic("c4", "no_such_kernel") == (None, None)
    assert bench.committed_traffic("c9", "gemm") == (None, None)


def test_dominant_kernel_names_the_kernel_the_library_launches():
    """The name fragments must exist in the committed summaries of the same workloads (they are what the
    traffic figure is looked up by)."""
    for name in ("c2", "c3", "c4", "c5"):
        cfg = W.CONFIGS[name]
        _, _, label, match = bench.dominant_kernel(cfg, None, {"gateup": 1.0}, 0)
        assert "gemm_tiled_kernel" in match, (name, match)
        text = open(os.path.join(ROOT, "profiles", f"verify_step_{name}.txt")).read()
        assert match in text, (name, match)
    one_row = W.scaled(W.CONFIGS["c2"], name="one_row", B=1, k=1, C=64)
    assert "gemm_tiled_kernel<2, 4, 1>" == bench.dominant_kernel(one_row, None, {"gateup": 1.0}, 0)[3]


def test_thresholds_are_the_frozen_calibrated_ones():
    lam = bench.golden_lambdas()
    want = np.loadtxt(os.path.join(ROOT, "tests", "golden", "lambdas_8b_final.txt"), comments="#").ravel()
    assert np.allclose(np.asarray(lam, dtype=float).ravel()[:3], want[:3])


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
