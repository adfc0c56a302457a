"""GPU parity of dsd_accept against the oracle on synthetic rows: ragged vocabulary sizes that span
one to many slices, chains and trees, strict / adaptive / forced relaxation, and the degenerate
cases (everything accepted, first token rejected, zero-mass draft entries)."""
import numpy as np
import pytest
import torch

from oracle import dsd_oracle as O
from paper_2511_11733_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def make_rows(seed, B, k, V, parent=None, spread=1.28, noise=0.5, zero_frac=0.0):
    rng = np.random.default_rng(seed)
    lg = (rng.standard_normal((B, k + 1, V)) * spread).astype(np.float32)
    dl = lg.astype(np.float64) + noise * rng.standard_normal((B, k + 1, V))
    q = np.exp(dl - dl.max(-1, keepdims=True))
    if zero_frac > 0:
        q[rng.random(q.shape) < zero_frac] = 0.0
    q = (q / q.sum(-1, keepdims=True)).astype(np.float32)
    par = list(range(k)) if parent is None else [int(p) for p in parent]
    toks = np.zeros((B, k), dtype=np.int32)
    for b in range(B):
        used = {}
        for i in range(1, k + 1):
            p = par[i - 1]
            qq = q[b, p].astype(np.float64).copy()
            for t in used.get(p, []):          # siblings are drawn without replacement
                qq[t] = 0.0
            t = int(rng.choice(V, p=qq / qq.sum()))
            used.setdefault(p, []).append(t)
            toks[b, i - 1] = t
    u = rng.random((B, k + 1)).astype(np.float32)
    return lg, q, toks, u


def run_case(ctx, lg, q, toks, parent, u, prm, what, tau_override=None, max_flagged_fraction=None, ratio_rtol=None):
    ora = O.accept(lg.astype(np.float64), q.astype(np.float64), toks, parent, u, H.oracle_prm(O, prm),
                   None if tau_override is None else tau_override.astype(np.float64))
    g = H.gpu_accept(ctx, torch.from_numpy(lg).to("cuda:0"), torch.from_numpy(q).to("cuda:0"), toks, parent, u, prm,
                     tau_override)
    st = H.compare_accept(g, ora, what, H.AcceptInputs(O, lg, q, toks, parent, u, prm, tau_override),
                          max_flagged_fraction=max_flagged_fraction)
    excused, near = st["excused_sequences"], st["flagged_accept"] + st["flagged_key"] + st["flagged_draw"]
    fin = np.isfinite(ora.ratio)
    # The reported ratios are fp64 over fp32 per-id terms: 1e-6 relative for the per-node rules.  In the
    # lossless walk a later sibling's p is a residual max(0, p - q) / Z; a Z of 0.05 or more is summed from
    # fp32 terms whose absolute error is ~1e-7 of p, so its relative error stays below 1e-7 / 0.05 (the
    # default bound here is looser than that needs); a smaller Z is summed again in fp64 (its own test
    # asks for 1e-6).  Decisions are protected by the oracle's near-tie margin of 1e-3 on the same ratio.
    if ratio_rtol is None:
        ratio_rtol = 2e-5 if prm.get("tree_mode", 0) == 2 else 1e-6
    np.testing.assert_allclose(g["ratio"][fin], ora.ratio[fin], rtol=ratio_rtol, err_msg=what)
    if prm.get("norm_match_kind", 0) == 1:      # a vocabulary-wide sum: fp32 terms on the GPU
        np.testing.assert_allclose(g["norm_match"], ora.norm_match, rtol=1e-6, err_msg=what)
    else:
        np.testing.assert_array_equal(g["norm_match"], ora.norm_match, err_msg=what)
    return ora, g, excused, near


@pytest.fixture(scope="module")
def ctx():
    return H.D.Context(0)


@pytest.mark.parametrize("V", [17, 2048, 2049, 5000, 128256, 262147])
def test_chain_strict_and_adaptive(ctx, V):
    B, k = (6, 5) if V > 10000 else (24, 5)
    lg, q, toks, u = make_rows(V, B, k, V)
    ora, g, ex, near = run_case(ctx, lg, q, toks, None, u, dict(tau=0.0), f"strict V={V}")
    assert 0 < ora.accepted_len.mean() < k
    # thresholds at the quartiles of this batch, so both branches of the key rule are taken
    with np.errstate(divide="ignore"):
        pt = np.stack([[O.softmax_row(lg[b, i], 1.0) for i in range(k + 1)] for b in range(B)])
    bi, ii = np.meshgrid(np.arange(B), np.arange(k), indexing="ij")
    pty, qy = pt[bi, ii, toks], q.astype(np.float64)[bi, ii, toks]
    l1 = float(np.quantile(np.log(qy) / np.log(pty), 0.75))
    l2 = float(np.quantile(np.abs(pty - qy), 0.75))
    prm = dict(tau=0.2, lambda1=l1, lambda2=l2, lambda3=0.2, top_m=min(8, V))
    ora, g, ex, near = run_case(ctx, lg, q, toks, None, u, prm, f"adaptive V={V}")
    assert 0.1 < ora.key.mean() < 0.9
    print(f"V={V}: key fraction {ora.key.mean():.2f}, mean accepted {ora.accepted_len.mean():.2f}, near ties {near}, excused {ex}")


@pytest.mark.parametrize("spread,noise", [(4.0, 0.5), (8.0, 2.0)])
def test_peaked_rows(ctx, spread, noise):
    """Rows like a trained model's: a few ids carry most of the mass (logit spread 4 and 8 standard
    deviations: top probability 0.1 .. 0.9), most probabilities underflow towards zero, accepted lengths are
    long.  Strict, adaptive and lossless-tree rules."""
    B, k, V = 6, 6, 50257
    lg, q, toks, u = make_rows(int(spread * 10), B, k, V, spread=spread, noise=noise)
    ora, *_ = run_case(ctx, lg, q, toks, None, u, dict(tau=0.0), f"peaked {spread} strict")
    run_case(ctx, lg, q, toks, None, u, dict(tau=0.3, lambda1=1.2, lambda2=1e-2, lambda3=0.5), f"peaked {spread} adaptive")
    parent = W.ranked_tree_parents((3, 2), 6)
    lg2, q2, toks2, u2 = make_rows(int(spread * 10) + 1, B, k, V, parent=parent, spread=spread, noise=noise)
    run_case(ctx, lg2, q2, toks2, parent, u2, dict(tau=0.0, tree_mode=2), f"peaked {spread} lossless tree")
    print(f"spread {spread}: top probability {np.exp(lg[0, 0] - lg[0, 0].max()).max() / np.exp(lg[0, 0] - lg[0, 0].max()).sum():.2f}, "
          f"mean accepted {ora.accepted_len.mean():.2f} of {k}")


def test_top_m_limits_and_temperature(ctx):
    lg, q, toks, u = make_rows(5, 8, 3, 3000)
    for top_m in (1, 16):
        run_case(ctx, lg, q, toks, None, u, dict(tau=0.3, lambda3=0.5, top_m=top_m), f"top_m={top_m}")
    run_case(ctx, lg, q, toks, None, u, dict(tau=0.3, temperature=0.7), "temperature")


def test_heavy_ties_in_the_top_m_selection(ctx):
    """Rows quantised to a handful of levels: hundreds of equal values in every slice of 2048 ids, so the
    per-slice threshold lets more ids through than the candidate list holds and the selection falls
    back to rounds over all ids.  Equal values go to the lower id on both sides, so NormMatch (compared
    exactly in run_case) and every decision not flagged as a near tie must agree."""
    B, k, V = 6, 4, 5000
    lg, q, toks, u = make_rows(21, B, k, V)
    lg = np.round(lg).astype(np.float32)
    dl = np.round(np.log(q.astype(np.float64)))
    q = np.exp(dl - dl.max(-1, keepdims=True))
    q = (q / q.sum(-1, keepdims=True)).astype(np.float32)
    assert len(np.unique(lg[0, 0])) < 16 and len(np.unique(q[0, 0])) < 32
    for top_m in (1, 8, 16):
        run_case(ctx, lg, q, toks, None, u, dict(tau=0.2, lambda3=0.3, top_m=top_m), f"quantised rows, top_m={top_m}")
    # ties in the target row only: the draft row keeps the candidate-list path
    lg2, q2, toks2, u2 = make_rows(22, B, k, V)
    run_case(ctx, np.round(lg2).astype(np.float32), q2, toks2, None, u2, dict(tau=0.2, lambda3=0.3), "quantised target rows")


def test_degenerate_cases(ctx):
    lg, q, toks, u = make_rows(9, 8, 4, 4100)
    # everything accepted -> bonus token from the last row
    u0 = u.copy(); u0[:, 1:] = 0.0
    ora, *_ = run_case(ctx, lg, q, toks, None, u0, dict(tau=0.0), "all accepted")
    assert (ora.accepted_len == 4).all()
    # first token rejected
    u1 = u.copy(); u1[:, 1] = np.float32(1 - 2 ** -24)
    q1 = q.copy()
    for b in range(8):
        q1[b, 0, toks[b, 0]] = 0.9            # make p/q tiny for the first token
    ora, *_ = run_case(ctx, lg, q1, toks, None, u1, dict(tau=0.0), "first rejected")
    assert (ora.accepted_len == 0).all()
    # tau = 1 accepts everything; draft == target accepts everything
    ora, *_ = run_case(ctx, lg, q, toks, None, u, dict(tau=1.0), "tau=1")
    assert (ora.accepted_len == 4).all()
    qt = np.stack([[O.softmax_row(lg[b, i], 1.0) for i in range(5)] for b in range(8)]).astype(np.float32)
    run_case(ctx, lg, qt, toks, None, u, dict(tau=0.0), "draft == target (fp32-rounded)")
    # draft rows with exact zeros (top-k style drafts)
    lgz, qz, tz, uz = make_rows(10, 8, 4, 3000, zero_frac=0.6)
    run_case(ctx, lgz, qz, tz, None, uz, dict(tau=0.25), "zero-mass draft entries")
    # k = 1
    lg1, q1, t1, u1 = make_rows(11, 16, 1, 777)
    run_case(ctx, lg1, q1, t1, None, u1, dict(tau=0.0), "k=1")


def test_forced_relaxation_per_node(ctx):
    lg, q, toks, u = make_rows(12, 12, 6, 2500)
    to = np.random.default_rng(0).choice([0.0, 0.1, 0.5, 1.0], size=(12, 6)).astype(np.float32)
    run_case(ctx, lg, q, toks, None, u, dict(tau=0.9), "tau_override", tau_override=to)


@pytest.mark.parametrize("mode", [0, 1])
def test_trees(ctx, mode):
    parent = W.ranked_tree_parents()
    k = len(parent)
    lg, q, toks, u = make_rows(13, 6, k, 6000, parent=parent)
    ora, g, ex, near = run_case(ctx, lg, q, toks, parent, u, dict(tau=0.2, lambda3=0.3, tree_mode=mode), f"tree mode {mode}")
    assert ora.accepted_len.max() >= 2
    small = [0, 0, 1, 1, 2]
    lg, q, toks, u = make_rows(14, 40, 5, 300, parent=small)
    run_case(ctx, lg, q, toks, small, u, dict(tau=0.0, tree_mode=mode), f"small tree mode {mode}")


def test_lossless_tree_rule(ctx):
    """DSD_TREE_LOSSLESS: recursive rejection over siblings drawn without replacement."""
    parent = W.ranked_tree_parents()
    k = len(parent)
    lg, q, toks, u = make_rows(21, 6, k, 6000, parent=parent)
    ora, g, ex, near = run_case(ctx, lg, q, toks, parent, u, dict(tau=0.2, lambda3=0.3, tree_mode=2), "lossless 32-node tree")
    assert ora.accepted_len.max() >= 2
    assert (ora.node_accept.sum(1) >= ora.accepted_len).all()
    # many rejections per level: a bushy tree under a poor draft
    bushy = [0] * 6 + [1] * 3 + [2] * 3
    lg, q, toks, u = make_rows(22, 24, len(bushy), 300, parent=bushy, noise=2.0)
    ora, *_ = run_case(ctx, lg, q, toks, bushy, u, dict(tree_mode=2), "lossless bushy tree")
    assert (ora.accepted_len == 0).any() and (ora.accepted_len > 0).any()
    # a chain gives the strict chain rule
    lg, q, toks, u = make_rows(23, 10, 7, 2500)
    ora, g, *_ = run_case(ctx, lg, q, toks, None, u, dict(tree_mode=2), "lossless chain")
    strict = O.accept(lg.astype(np.float64), q.astype(np.float64), toks, None, u, H.oracle_prm(O, dict(tau=0.0)))
    np.testing.assert_array_equal(g["accepted_len"], strict.accepted_len)
    np.testing.assert_array_equal(g["next_token"], strict.next_token)
    # draft rows with exact zeros, full-size vocabulary
    lg, q, toks, u = make_rows(24, 2, 10, 128256, parent=W.ranked_tree_parents((3, 2, 2), 10), zero_frac=0.5)
    run_case(ctx, lg, q, toks, W.ranked_tree_parents((3, 2, 2), 10), u, dict(tree_mode=2), "lossless, vocabulary 128256")


@pytest.mark.parametrize("noise", [0.02, 0.05])
def test_lossless_walk_with_a_draft_close_to_the_target_on_peaked_rows(ctx, noise):
    """A good draft on rows like a trained model's: target and draft differ by a few per mille of total
    variation, so after a rejection the next sibling is tested against a residual divided by a Z of 1e-3 .. 1e-2.
    The walk sums such a Z again in fp64 with the row renormalised in fp64; ratios then agree with the oracle
    to 1e-6 like everywhere else and no sequence needs the near-tie exception."""
    parent = W.ranked_tree_parents((3, 2, 2), 10)
    B, k, V = 8, len(parent), 50257
    lg, q, toks, u = make_rows(int(noise * 1000), B, k, V, parent=parent, spread=6.0, noise=noise)
    # make rejections happen although the draft is good: uniforms close to 1 for the first child of every node
    u[:, 1:] = 1.0 - (1.0 - u[:, 1:]) * 0.02
    ora, g, ex, near = run_case(ctx, lg, q, toks, parent, u, dict(tree_mode=2), f"lossless, draft noise {noise}", ratio_rtol=1e-6)
    tested = ora.ratio != 0
    assert ex == 0 and (~ora.node_accept[tested]).sum() >= 4, "the case must contain rejections"
    pt = O.softmax_row(lg[0, 0].astype(np.float64), 1.0)
    z = np.maximum(pt - q[0, 0].astype(np.float64), 0).sum()
    print(f"noise {noise}: residual mass of a root row {z:.2e}, rejections {int((~ora.node_accept[tested]).sum())}")
    assert z < 0.05


def test_greedy_verification_at_temperature_zero(ctx):
    rng = np.random.default_rng(41)
    for what, parent, B, V in (("chain", None, 9, 5000), ("tree", W.ranked_tree_parents(), 5, 128256),
                               ("small tree", [0, 0, 1, 1, 2], 30, 300)):
        k = 6 if parent is None else len(parent)
        lg, q, toks, u = make_rows(int(rng.integers(1 << 30)), B, k, V, parent=parent)
        par = list(range(k)) if parent is None else [int(p) for p in parent]
        for b in range(B):                    # most drafts hit the arg max of their parent's row, some do not
            for i in range(1, k + 1):
                if rng.random() < 0.7:
                    toks[b, i - 1] = int(np.argmax(lg[b, par[i - 1]]))
        lg[0, 0, 7] = lg[0, 0].max()          # a tie in the root row of sequence 0: the lower id wins
        lg[0, 0, 3] = lg[0, 0, 7]
        for mode in (0, 1, 2):
            ora, g, ex, near = run_case(ctx, lg, q, toks, parent, u, dict(temperature=0.0, tree_mode=mode), f"greedy {what} mode {mode}")
            assert ex == 0 and ora.accepted_len.max() >= 2
    # draft_probs and uniforms may be NULL
    t = torch.from_numpy(lg).to("cuda:0")
    tk = torch.from_numpy(toks).to("cuda:0")
    pr = torch.from_numpy(np.asarray(par, dtype=np.int32)).to("cuda:0")
    alen = torch.zeros(B, dtype=torch.int32, device="cuda:0")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda:0")
    H.D.dsd_accept(ctx, t, None, tk, pr, None, H.D.accept_params(temperature=0.0), B, k, V, alen, nxt, None)
    torch.cuda.synchronize()
    ora = O.accept(lg.astype(np.float64), q.astype(np.float64), toks, par, u, O.AcceptParams(temperature=0.0))
    np.testing.assert_array_equal(alen.cpu().numpy(), ora.accepted_len)
    np.testing.assert_array_equal(nxt.cpu().numpy(), ora.next_token)


def test_key_rule_variants_and_tau_sweep(ctx):
    """Overlap reading of NormMatch, row-entropy reading of the first criterion, and the accept rate as
    tau grows (the trade-off of the paper's ablation), GPU against oracle."""
    parent = W.ranked_tree_parents((3, 2, 2), 10)
    for what, par, B, k, V in (("chain", None, 24, 6, 5000), ("tree", parent, 12, 10, 128256)):
        lg, q, toks, u = make_rows(71 if par is None else 72, B, k, V, parent=par)
        probe = O.accept(lg.astype(np.float64), q.astype(np.float64), toks, par, u,
                         H.oracle_prm(O, dict(norm_match_kind=1, entropy_kind=1)))
        lam3 = float(np.median(probe.norm_match))                       # about half of the rows below it
        pl = [int(p) for p in (range(k) if par is None else par)]
        ratios = []
        for b in range(B):
            for p_row in set(pl):
                pt = O.softmax_row(lg[b, p_row].astype(np.float64), 1.0)
                ratios.append(O.row_entropy(q[b, p_row].astype(np.float64)) / O.row_entropy(pt))
        lam1 = float(np.median(ratios))
        for prm in (dict(tau=0.3, lambda3=lam3, norm_match_kind=1), dict(tau=0.3, lambda1=lam1, entropy_kind=1),
                    dict(tau=0.3, lambda1=lam1, lambda3=lam3, norm_match_kind=1, entropy_kind=1, tree_mode=1),
                    dict(lambda3=lam3, norm_match_kind=1, tree_mode=2)):
            # lambda1 sits at the median of the rows' entropy ratios, which on these near-flat rows all lie within
            # a percent of each other: a large share of the nodes is within 1e-3 of that threshold by construction
            ora, g, ex, near = run_case(ctx, lg, q, toks, par, u, prm, f"{what} {prm}",
                                        max_flagged_fraction=0.5 if prm.get("entropy_kind") else None)
            assert 0.1 < ora.key.mean() < 0.9, (what, prm, ora.key.mean())
    # accept rate against tau, no key tokens
    lg, q, toks, u = make_rows(73, 64, 5, 3000, noise=1.0)
    rates = []
    for tau in (0.0, 0.1, 0.2, 0.4, 0.8):
        ora, g, ex, near = run_case(ctx, lg, q, toks, None, u, dict(tau=tau), f"tau {tau}")
        rates.append(float(g["node_accept"].mean()))
    print("accept rate of a node against tau (0, .1, .2, .4, .8):", [round(r, 3) for r in rates])
    assert all(b >= a for a, b in zip(rates, rates[1:])) and rates[-1] > rates[0] + 0.1


def test_k_max_chain(ctx):
    lg, q, toks, u = make_rows(15, 2, 64, 1000, noise=0.1)
    ora, *_ = run_case(ctx, lg, q, toks, None, u, dict(tau=0.3), "k=64")
    assert ora.accepted_len.max() > 8


def test_argument_errors(ctx):
    t = torch.zeros((1, 2, 10), dtype=torch.float32, device="cuda:0")
    i = torch.zeros((1, 1), dtype=torch.int32, device="cuda:0")
    with pytest.raises(H.D.DsdError):
        H.D.dsd_accept(ctx, t, t, i, None, t, H.D.accept_params(top_m=17), 1, 1, 10, i, i)
    with pytest.raises(H.D.DsdError):
        H.D.dsd_accept(ctx, t, t, i, None, t, H.D.accept_params(tau=1.5), 1, 1, 10, i, i)
    with pytest.raises(H.D.DsdError):
        H.D.dsd_accept(ctx, t, t, i, None, t, H.D.accept_params(), 1, 65, 10, i, i)
