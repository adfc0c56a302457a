"""Writes tests/golden/lambdas_8b_final.txt: thresholds of the key-token rule for the
final-stage workloads.  The paper calibrates lambda_1..3 "on a small validation set" and prints
no values (section 2.3); here they are quantiles over a seeded synthetic calibration batch with
the statistics of the benchmark rows (target logits ~ N(0, (0.02 sqrt(d))^2) over the vocabulary,
draft logits = target + N(0, 0.5^2), drafted token ~ draft row):
    lambda1 = 75th percentile of H_d/H_t, lambda2 = 75th percentile of |P_t(y) - q(y)|,
    lambda3 = 25th percentile of NormMatch (top_m = 8), nudged so that the strict '<' test fires.
Uses only oracle/ and the input generators.  Run from the repository root:
    python tests/golden/calibrate_lambdas.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import dsd_oracle as O  # noqa: E402
from paper_2511_11733_amd import workloads as W  # noqa: E402


def main():
    cfg = W.CONFIGS["c3"]
    m = cfg.model
    n = 256
    lg = W.normal(cfg.seed, W.STREAM_CALIB, "calib.logits", (n, m.V), W.kv_std(m))
    nz = W.normal(cfg.seed, W.STREAM_CALIB, "calib.noise", (n, m.V), cfg.noise_std)
    u = W.rng_for(cfg.seed, W.STREAM_CALIB, "calib.u").random(n)
    ratio, diff, nm = [], [], []
    for i in range(n):
        pt = O.softmax_row(lg[i], 1.0)
        q = O.softmax_row(lg[i].astype(np.float64) + nz[i], 1.0).astype(np.float32).astype(np.float64)
        y = W.draw_categorical(q, float(u[i]))
        ratio.append(np.log(q[y]) / np.log(pt[y]))
        diff.append(abs(pt[y] - q[y]))
        nm.append(O.norm_match(pt, q, cfg.top_m))
    l1 = float(np.quantile(ratio, 0.75))
    l2 = float(np.quantile(diff, 0.75))
    l3 = float(np.quantile(nm, 0.25)) + 0.5 / cfg.top_m
    key = [(r > l1) or (d > l2) or (x < l3) for r, d, x in zip(ratio, diff, nm)]
    out = os.path.join(ROOT, "tests", "golden", "lambdas_8b_final.txt")
    with open(out, "w") as f:
        f.write(f"{l1!r} {l2!r} {l3!r}\n")
        f.write("# lambda1 lambda2 lambda3 for top_m = 8, tau = 0.2; written by calibrate_lambdas.py\n")
        f.write(f"# key fraction on the calibration batch: {np.mean(key):.3f}; NormMatch quartiles "
                f"{np.quantile(nm, [0.25, 0.5, 0.75]).tolist()}\n")
    print(open(out).read())


if __name__ == "__main__":
    main()
