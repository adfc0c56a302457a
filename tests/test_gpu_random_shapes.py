"""GPU: seeded random problems against the oracle.  The hand-picked cases of the other files aim at
known boundaries (tile counts, slice counts, ragged tails); these sweep combinations nobody thought of:
row counts, ragged lengths including empty contexts, chains and trees, GQA group sizes, model widths on
and off the panel path for the verify step; vocabulary sizes around the slice size, tree modes, key-rule
readings, temperatures, peaked and flat rows, zero-mass draft entries for dsd_accept."""
import numpy as np
import pytest

from paper_2511_11733_amd import workloads as W
from tests import helpers as H
from tests.test_gpu_accept import make_rows, run_case
from tests.test_gpu_bf16 import check, mini

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12])
def test_random_verify_steps(seed):
    rng = np.random.default_rng(seed)
    for it in range(30):
        k = int(rng.choice([1, 2, 3, 5, 7, 8, 12, 16, 20, 32]))
        B = int(rng.integers(1, max(1, min(12, 128 // k)) + 1))
        lens = [int(rng.integers(0, 300)) for _ in range(B)]
        head = bool(rng.integers(0, 2))
        tree = ((3, 2, 2, 2, 1, 1), k) if (k >= 5 and rng.integers(0, 2)) else None
        Hq, Hkv = [(8, 2), (8, 8), (16, 2), (4, 1)][int(rng.integers(0, 4))]
        d = int(rng.choice([512, 1024]))
        F = int(rng.choice([1536, 2048, 1792]))
        name = f"rnd{seed}_{it}_B{B}k{k}_H{Hq}_{Hkv}_d{d}_F{F}_{'tree' if tree else 'chain'}_{'head' if head else 'mid'}"
        check(mini(name, B=B, k=k, lens=lens, tree=tree, head=head, V=4112, L=1, Hq=Hq, Hkv=Hkv, d=d, F=F))


@pytest.mark.parametrize("seed", [21, 22])
def test_random_accept_problems(seed):
    rng = np.random.default_rng(seed)
    ctx = H.D.Context(0)
    for it in range(40):
        V = int(rng.choice([17, 64, 300, 2047, 2048, 2049, 4097, 9000, 33000]))
        B = int(rng.integers(1, 7))
        k = int(rng.integers(1, 13))
        parent = W.ranked_tree_parents((3, 2, 2, 1, 1, 1), k) if (k >= 4 and rng.integers(0, 2)) else None
        spread = float(rng.choice([0.5, 1.28, 3.0, 6.0]))
        noise = float(rng.choice([0.1, 0.5, 1.5]))
        zero_frac = float(rng.choice([0.0, 0.0, 0.5]))
        prm = dict(tau=float(rng.choice([0.0, 0.2, 0.6, 1.0])), lambda1=float(rng.choice([0.9, 1.05, 1.5])),
                   lambda2=float(rng.choice([1e-4, 1e-2, 0.2])), lambda3=float(rng.choice([0.1, 0.3, 0.8])),
                   top_m=int(min(V, rng.integers(1, 17))), temperature=float(rng.choice([1.0, 0.7, 1.3])),
                   tree_mode=int(rng.integers(0, 3)), norm_match_kind=int(rng.integers(0, 2)),
                   entropy_kind=int(rng.integers(0, 2)))
        what = f"rnd{seed}_{it} V={V} B={B} k={k} {'tree' if parent is not None else 'chain'} spread={spread} {prm}"
        lg, q, toks, u = make_rows(seed * 1000 + it, B, k, V, parent=parent, spread=spread, noise=noise, zero_frac=zero_frac)
        run_case(ctx, lg, q, toks, parent, u, prm, what)
