"""Pins for the oracle's near-tie flags and for the comparison rule built on them (CPU only).

The accept parity tests tolerate exactly one kind of difference between the HIP path and the
oracle: a decision the oracle marks as a near tie, for that node and that kind of decision.  An
over-eager flag would silently hollow those tests out, so the flags themselves are pinned here on
constructed cases: for every class one case that must be flagged and one just outside the band that
must not, always at one node only.  The second half plants differences into a copy of the oracle's
own result (never into the GPU path) and checks that the comparison rule accepts what it should
and nothing else."""
import copy

import numpy as np
import pytest

from oracle import dsd_oracle as O
from tests import helpers as H


def softmax(z):
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max(-1, keepdims=True))
    return e / e.sum(-1, keepdims=True)


def chain_case(seed=0, B=1, k=3, V=7):
    """Small chain with generic rows: nothing near any threshold unless a test moves it there."""
    rng = np.random.default_rng(seed)
    lg = rng.standard_normal((B, k + 1, V)) * 1.5
    q = softmax(lg + 0.7 * rng.standard_normal((B, k + 1, V)))
    toks = rng.integers(0, V, size=(B, k)).astype(np.int32)
    u = rng.random((B, k + 1)) * 0.5 + 0.25
    return lg, q, toks, u


# ------------------------------------------------------------------------------- the flags
@pytest.mark.parametrize("delta,flag", [(5e-4, True), (-5e-4, True), (2e-3, False), (-2e-3, False)])
def test_accept_tie_is_flagged_within_1e_3_of_the_uniform_at_that_node_only(delta, flag):
    lg, q, toks, u = chain_case(1)
    pt = softmax(lg)
    # make node 2's ratio p/q fall below 1, then put its uniform at ratio - delta
    y = int(toks[0, 1])
    q[0, 1, y] = max(q[0, 1, y], 2.0 * pt[0, 1, y])
    ratio = pt[0, 1, y] / q[0, 1, y]
    u[0, 2] = ratio - delta
    # the other nodes stay far from their ratios
    for i in (1, 3):
        yi = int(toks[0, i - 1])
        ri = min(pt[0, i - 1, yi] / q[0, i - 1, yi], 1.0)
        u[0, i] = ri * 0.5
    out = O.accept(lg, q, toks, None, u, O.AcceptParams())
    assert out.tie_accept[0].tolist() == [False, flag, False]
    assert out.node_accept[0, 1] == (delta > 0)          # u below the ratio accepts
    assert bool(out.near_tie[0] & 1) == flag


@pytest.mark.parametrize("rel,flag", [(5e-4, True), (-5e-4, True), (3e-3, False), (-3e-3, False)])
def test_key_tie_lambda1_and_lambda2_bands(rel, flag):
    lg, q, toks, u = chain_case(12)
    pt = softmax(lg)
    y = int(toks[0, 1])
    h_t, h_d = -np.log(pt[0, 1, y]), -np.log(q[0, 1, y])
    # criterion 1 of node 2 at relative distance rel from its threshold; the other nodes' ratios differ
    # from node 2's by far more than the band (generic rows)
    lam1 = h_d / h_t / (1.0 + rel)
    out = O.accept(lg, q, toks, None, u, O.AcceptParams(lambda1=lam1, tau=0.2))
    others = [abs(-np.log(q[0, i, int(toks[0, i])]) / -np.log(pt[0, i, int(toks[0, i])]) / lam1 - 1.0) for i in (0, 2)]
    assert min(others) > 1e-2
    assert out.tie_key[0].tolist() == [False, flag, False]
    assert out.key[0, 1] == (rel > 0)                     # H_d = lam1 H_t (1 + rel) > lam1 H_t
    # criterion 2
    gap = abs(pt[0, 1, y] - q[0, 1, y])
    lam2 = gap / (1.0 + rel)
    out = O.accept(lg, q, toks, None, u, O.AcceptParams(lambda2=lam2, tau=0.2))
    assert out.tie_key[0].tolist() == [False, flag, False]
    assert out.key[0, 1] == (rel > 0)
    assert bool(out.near_tie[0] & 2) == flag


@pytest.mark.parametrize("rel_gap,flag", [(1e-6, True), (1e-3, False)])
def test_key_tie_top_m_boundary_gap_flags_every_child_of_that_row(rel_gap, flag):
    # tree: nodes 1 and 2 hang under the root, node 3 under node 1; M = 2
    parent = [0, 0, 1]
    V = 6
    base = np.array([0.30, 0.25, 0.20, 0.12, 0.08, 0.05])
    rows_p = np.tile(base, (4, 1))
    # root row of the target: second and third largest differ by rel_gap (relative), straddling M = 2
    rows_p[0] = np.array([0.40, 0.20, 0.20 * (1.0 - rel_gap), 0.10, 0.06, 0.04])
    rows_p /= rows_p.sum(-1, keepdims=True)
    lg = np.log(rows_p)[None]
    q = np.tile(np.array([0.28, 0.24, 0.18, 0.14, 0.09, 0.07]), (1, 4, 1))
    toks = np.array([[0, 3, 1]], dtype=np.int32)
    u = np.full((1, 4), 0.5)
    out = O.accept(lg, q, toks, parent, u, O.AcceptParams(lambda3=0.6, top_m=2, tau=0.1))
    assert out.tie_key[0].tolist() == [flag, flag, False]


def test_key_tie_overlap_reading_near_lambda3():
    lg, q, toks, u = chain_case(3)
    nm = O.norm_match_overlap(softmax(lg)[0, 1], q[0, 1])
    for d, flag in ((5e-7, True), (-5e-7, True), (1e-4, False)):
        out = O.accept(lg, q, toks, None, u, O.AcceptParams(lambda3=nm + d, norm_match_kind=O.NM_OVERLAP, tau=0.1))
        assert out.tie_key[0].tolist() == [False, flag, False]


@pytest.mark.parametrize("rel,flag", [(1e-7, True), (-1e-7, True), (1e-3, False)])
def test_draw_tie_is_flagged_within_1e_6_of_a_cdf_boundary(rel, flag):
    lg, q, toks, u = chain_case(4)
    pt = softmax(lg)
    u[0, 1] = 0.999999                                    # first node rejected whenever its ratio is below 1
    y = int(toks[0, 0])
    q[0, 0, y] = max(q[0, 0, y], 3.0 * pt[0, 0, y])
    q[0, 0] /= q[0, 0].sum()
    w = np.maximum(pt[0, 0] - q[0, 0], 0.0)
    c = np.cumsum(w)
    assert (w > 0).sum() >= 2
    j = int(np.nonzero(w > 0)[0][0])                      # an interior boundary: more mass follows
    u[0, 0] = c[j] / c[-1] * (1.0 + rel)
    out = O.accept(lg, q, toks, None, u, O.AcceptParams())
    assert out.accepted_len[0] == 0
    assert bool(out.tie_draw[0]) == flag and bool(out.near_tie[0] & 4) == flag
    if rel < 0:
        assert out.next_token[0] == j                     # just below the boundary: still id j
    elif flag:
        assert out.next_token[0] > j


def test_flags_are_rare_on_generic_rows():
    """2 * 1e-3 wide bands: a few per thousand decisions, not a few per ten."""
    rng = np.random.default_rng(7)
    B, k, V = 60, 6, 400
    lg = rng.standard_normal((B, k + 1, V)) * 1.3
    q = softmax(lg + 0.5 * rng.standard_normal((B, k + 1, V)))
    toks = np.array([[rng.choice(V, p=q[b, i]) for i in range(k)] for b in range(B)], dtype=np.int32)
    u = rng.random((B, k + 1))
    pt = softmax(lg)
    bi, ii = np.meshgrid(np.arange(B), np.arange(k), indexing="ij")
    l1 = float(np.quantile(np.log(q[bi, ii, toks]) / np.log(pt[bi, ii, toks]), 0.75))
    l2 = float(np.quantile(np.abs(pt[bi, ii, toks] - q[bi, ii, toks]), 0.75))
    out = O.accept(lg, q, toks, None, u, O.AcceptParams(lambda1=l1, lambda2=l2, lambda3=0.3, tau=0.2))
    n = B * k
    assert out.tie_accept.sum() <= 0.02 * n, out.tie_accept.sum()
    assert out.tie_key.sum() <= 0.05 * n, out.tie_key.sum()
    assert out.tie_draw.sum() <= 1


def test_forced_decision_is_followed_downstream():
    lg, q, toks, u = chain_case(5)
    u[0, 1:] = 0.0                                        # everything accepted
    base = O.accept(lg, q, toks, None, u, O.AcceptParams())
    assert base.accepted_len[0] == 3
    fa = np.array([[-1, 0, -1]])
    out = O.accept(lg, q, toks, None, u, O.AcceptParams(), force_accept=fa)
    assert out.accepted_len[0] == 1 and out.accepted_path[0].tolist() == [1, -1, -1]
    # the extra token now comes from the residual of row 1 (node 2 rejected there), by the oracle's own rule
    pt = softmax(lg)
    w = np.maximum(pt[0, 1] - q[0, 1], 0.0)
    tok, _ = O.inverse_cdf(w, u[0, 0])
    assert out.next_token[0] == tok
    # pinning the key flag changes tau of that node only
    fk = np.array([[-1, 1, -1]])
    out = O.accept(lg, q, toks, None, u, O.AcceptParams(tau=0.3), force_key=fk)
    assert out.tau_used[0].tolist() == [0.3, 0.0, 0.3] and out.key[0].tolist() == [False, True, False]


# ------------------------------------------------------------------------------- the comparison rule
def as_gpu(out):
    """An oracle result in the shape gpu_accept returns (what a perfect implementation would give)."""
    return dict(accepted_len=out.accepted_len.copy(), next_token=out.next_token.copy(),
                accepted_path=out.accepted_path.copy(), key=out.key.copy(), node_accept=out.node_accept.copy())


def near_tie_case():
    """Chain of 3, strict rule: node 2's uniform sits 5e-4 below its ratio (accepted, flagged)."""
    lg, q, toks, u = chain_case(6)
    pt = softmax(lg)
    u[0, 1:] = 0.0
    y = int(toks[0, 1])
    q[0, 1, y] = max(q[0, 1, y], 2.0 * pt[0, 1, y])
    u[0, 2] = pt[0, 1, y] / q[0, 1, y] - 5e-4
    prm = dict(tau=0.0)
    ora = O.accept(lg, q, toks, None, u, H.oracle_prm(O, prm))
    assert ora.tie_accept[0].tolist() == [False, True, False] and ora.accepted_len[0] == 3
    return H.AcceptInputs(O, lg, q, toks, None, u, prm), ora


def test_compare_identical_results_need_no_excuse():
    inp, ora = near_tie_case()
    st = H.compare_accept(as_gpu(ora), ora, "identical", inp, max_excused=0)
    assert st["excused_sequences"] == 0 and st["flagged_accept"] == 1


def test_compare_accepts_a_flagged_decision_falling_the_other_way_with_consistent_downstream():
    inp, ora = near_tie_case()
    other = inp.rerun(0, None, np.array([[-1, 0, -1]]))   # what follows when node 2 is rejected instead
    assert other.accepted_len[0] == 1
    st = H.compare_accept(as_gpu(other), ora, "flipped near tie", inp)
    assert st["excused_sequences"] == 1
    with pytest.raises(AssertionError):
        H.compare_accept(as_gpu(other), ora, "flipped near tie, none allowed", inp, max_excused=0)


def test_compare_rejects_a_difference_at_an_unflagged_node_even_if_another_node_is_flagged():
    inp, ora = near_tie_case()
    wrong = inp.rerun(0, None, np.array([[0, -1, -1]]))   # node 1 rejected: node 1 is not a near tie
    assert wrong.accepted_len[0] == 0
    with pytest.raises(AssertionError, match="not within 1e-3"):
        H.compare_accept(as_gpu(wrong), ora, "wrong at node 1", inp)


def test_compare_rejects_inconsistent_downstream_of_a_flagged_decision():
    inp, ora = near_tie_case()
    other = as_gpu(inp.rerun(0, None, np.array([[-1, 0, -1]])))
    other["next_token"] = (other["next_token"] + 1) % 7   # right decision flip, wrong extra token
    with pytest.raises(AssertionError):
        H.compare_accept(other, ora, "wrong token after the flip", inp)
    other = as_gpu(inp.rerun(0, None, np.array([[-1, 0, -1]])))
    other["accepted_len"] = other["accepted_len"] + 1
    with pytest.raises(AssertionError):
        H.compare_accept(other, ora, "wrong length after the flip", inp)


def test_compare_rejects_a_plain_wrong_token_or_length():
    inp, ora = near_tie_case()
    g = as_gpu(ora)
    g["next_token"] = (g["next_token"] + 1) % 7
    with pytest.raises(AssertionError):
        H.compare_accept(g, ora, "wrong token", inp)
    g = as_gpu(ora)
    g["accepted_len"] = g["accepted_len"] - 1
    with pytest.raises(AssertionError):
        H.compare_accept(g, ora, "wrong length", inp)


def test_compare_key_flag_flip_only_where_the_key_rule_is_near_its_threshold():
    lg, q, toks, u = chain_case(8)
    pt = softmax(lg)
    y = int(toks[0, 1])
    lam1 = (-np.log(q[0, 1, y])) / (-np.log(pt[0, 1, y])) / (1.0 + 5e-4)
    prm = dict(tau=0.3, lambda1=lam1)
    ora = O.accept(lg, q, toks, None, u, H.oracle_prm(O, prm))
    assert ora.tie_key[0].tolist() == [False, True, False] and ora.key[0, 1]
    inp = H.AcceptInputs(O, lg, q, toks, None, u, prm)
    flipped = inp.rerun(0, np.array([[-1, 0, -1]]), None)
    st = H.compare_accept(as_gpu(flipped), ora, "key flip at the flagged node", inp)
    assert st["excused_sequences"] == 1
    bad = inp.rerun(0, np.array([[1 - int(ora.key[0, 0]), -1, -1]]), None)
    with pytest.raises(AssertionError, match="without a key near tie"):
        H.compare_accept(as_gpu(bad), ora, "key flip at an unflagged node", inp)


def test_compare_draw_difference_only_with_a_draw_near_tie():
    lg, q, toks, u = chain_case(4)
    pt = softmax(lg)
    u[0, 1] = 0.999999
    y = int(toks[0, 0])
    q[0, 0, y] = max(q[0, 0, y], 3.0 * pt[0, 0, y])
    q[0, 0] /= q[0, 0].sum()
    w = np.maximum(pt[0, 0] - q[0, 0], 0.0)
    c = np.cumsum(w)
    pos = np.nonzero(w > 0)[0]
    j = int(pos[0])
    u[0, 0] = c[j] / c[-1] * (1.0 - 1e-7)
    prm = dict(tau=0.0)
    ora = O.accept(lg, q, toks, None, u, H.oracle_prm(O, prm))
    assert ora.tie_draw[0] and ora.next_token[0] == j
    inp = H.AcceptInputs(O, lg, q, toks, None, u, prm)
    g = as_gpu(ora)
    g["next_token"][0] = int(pos[1])                      # the neighbour across the boundary
    assert H.compare_accept(g, ora, "draw near tie", inp)["excused_sequences"] == 1
    u2 = u.copy()
    u2[0, 0] = c[j] / 2 / c[-1]                           # the middle of id j's interval
    ora2 = O.accept(lg, q, toks, None, u2, H.oracle_prm(O, prm))
    assert not ora2.tie_draw[0]
    g = as_gpu(ora2)
    g["next_token"][0] = (int(g["next_token"][0]) + 1) % 7
    with pytest.raises(AssertionError):
        H.compare_accept(g, ora2, "draw differs without a near tie", H.AcceptInputs(O, lg, q, toks, None, u2, prm))


def test_compare_refuses_an_excuse_that_covers_too_many_decisions():
    rng = np.random.default_rng(9)
    B, k, V = 10, 6, 50
    lg = rng.standard_normal((B, k + 1, V))
    q = softmax(lg + 0.5 * rng.standard_normal((B, k + 1, V)))
    toks = rng.integers(0, V, size=(B, k)).astype(np.int32)
    u = rng.random((B, k + 1))
    prm = dict(tau=0.0)
    ora = O.accept(lg, q, toks, None, u, H.oracle_prm(O, prm))
    inp = H.AcceptInputs(O, lg, q, toks, None, u, prm)
    H.compare_accept(as_gpu(ora), ora, "generic", inp, max_excused=0)
    eager = copy.deepcopy(ora)
    eager.tie_accept[:] = True                            # an oracle that flags everything
    with pytest.raises(AssertionError, match="excuse is too wide"):
        H.compare_accept(as_gpu(ora), eager, "over-eager flags", inp)


def test_lossless_walk_flip_is_followed_through_the_siblings():
    parent = [0, 0, 0, 1, 2]
    rng = np.random.default_rng(10)
    V = 9
    lg = rng.standard_normal((1, 6, V))
    q = softmax(lg + 0.8 * rng.standard_normal((1, 6, V)))
    toks = np.array([[0, 1, 2, 3, 4]], dtype=np.int32)
    u = rng.random((1, 6)) * 0.4 + 0.3
    pt = softmax(lg)
    q[0, 0, 0] = max(q[0, 0, 0], 2.0 * pt[0, 0, 0])
    q[0, 0] /= q[0, 0].sum()
    u[0, 1] = pt[0, 0, 0] / q[0, 0, 0] + 5e-4              # node 1 just rejected
    prm = dict(tree_mode=2)
    ora = O.accept(lg, q, toks, parent, u, H.oracle_prm(O, prm))
    assert ora.tie_accept[0, 0] and not ora.node_accept[0, 0]
    inp = H.AcceptInputs(O, lg, q, toks, parent, u, prm)
    other = inp.rerun(0, None, np.array([[1, -1, -1, -1, -1]]))
    assert other.accepted_path[0, 0] == 1
    st = H.compare_accept(as_gpu(other), ora, "lossless flip", inp)
    assert st["excused_sequences"] == 1
