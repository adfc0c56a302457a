"""CPU oracle for the DSD verify step and acceptance rule.  TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64 everywhere, no blocking, no fusion, no reordering.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this file; the product path
(the HIP library and its binding) never does, and shares no code with it.

What is computed, and where the paper fixes it:

* ``stage_forward``  -- the target model's single forward pass over the drafted rows
  (section 2.1, "the target verifies in a single forward pass"), restricted to the
  contiguous block of layers one node hosts (section 2.2).  The paper names the model
  families only (section 3.1: Llama3.1-8B, Qwen3-8B); the block below is the Llama
  decoder layer: pre-norm RMSNorm, rotary embedding in the rotate-half convention,
  grouped-query attention, SwiGLU FFN, no biases.
* ``accept``  -- the loop of Algorithm 1: key-token test (Eq. "Key", section 2.3), softened
  target  P~ = P_t^(1-tau) P_d^tau  renormalised over the vocabulary (section 2.3,
  "Verification scaling"), in-order verification with a break at the first rejection,
  then one additional token.  The accept test itself is the rule of the speculative
  sampling work the paper cites in section 2.1: accept with probability min(1, p/q);
  on rejection draw from the normalised positive part of (p - q); after a fully
  accepted window draw a bonus token from the target row.

Pins (tests/test_oracle_*.py): forward against an independent library implementation of
the same architecture and against closed forms; accept against exact enumeration,
chi-square Monte Carlo, the tau = 0 / tau = 1 limits of the softened target and the
closed-form expected accepted length.  The key-rule constants (lambda_1..3, top-M) have
no values in the paper: "parity unpinned" for their numeric choice (the rule's structure
is pinned).  The tree rule with more than one child per node is not in the paper and not
distribution preserving: "parity unpinned" beyond the degenerate tree and brute force
over paths.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

F64 = np.float64


# =============================================================================== inputs
def widen(a: np.ndarray) -> np.ndarray:
    """Any stored tensor -> float64.  uint16 arrays are bfloat16 bit patterns."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(F64)
    return a.astype(F64)


# =============================================================================== forward
def rms_norm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(v: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: element i pairs with element i + hd/2 and the
    pair is rotated by the angle pos * theta^(-2i/hd).   v: [..., rows, heads, hd],
    pos: [rows]."""
    hd = v.shape[-1]
    half = hd // 2
    inv_freq = theta ** (-np.arange(half, dtype=F64) * 2.0 / hd)
    ang = pos.astype(F64)[:, None] * inv_freq[None, :]          # [rows, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a = v[..., :half]
    b = v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def ancestor_matrix(parent: Sequence[int]) -> np.ndarray:
    """A[t, s] = True when node s+1 is node t+1 itself or one of its ancestors.
    parent[i-1] in 0..k is the parent of node i (0 = the root, i.e. the committed context).
    A chain (parent[i-1] = i-1) gives the lower-triangular causal mask."""
    k = len(parent)
    A = np.zeros((k, k), dtype=bool)
    for t in range(k):
        n = t + 1
        while n != 0:
            A[t, n - 1] = True
            n = int(parent[n - 1])
    return A


def node_depths(parent: Sequence[int]) -> np.ndarray:
    """Number of edges between node i and the first drafted level (children of root: 0)."""
    k = len(parent)
    d = np.zeros(k, dtype=np.int64)
    for t in range(k):
        n = int(parent[t])
        while n != 0:
            d[t] += 1
            n = int(parent[n - 1])
    return d


@dataclass
class StageOut:
    hidden: np.ndarray                 # [B, k, d]
    logits: Optional[np.ndarray]       # [B, k, V] on the final stage
    new_k: np.ndarray                  # [L, B, Hkv, k, hd]  rotated keys of the drafted rows
    new_v: np.ndarray                  # [L, B, Hkv, k, hd]
    taps: Dict[str, np.ndarray] = field(default_factory=dict)


def stage_forward(model, get_weight: Callable[[str], np.ndarray],
                  kv_k: Optional[np.ndarray], kv_v: Optional[np.ndarray], ctx_len: Sequence[int],
                  hidden_in: Optional[np.ndarray], tokens: Optional[np.ndarray],
                  parent: Optional[Sequence[int]] = None, want_taps: bool = False) -> StageOut:
    """One node's share of the verification pass over k drafted rows per sequence.

    model       object with L, d, Hq, Hkv, hd, F, V, has_embed, has_head, rope_theta, eps
    get_weight  name -> stored tensor (matrices [out, in]); called once per use so that a
                caller may produce layers one at a time
    kv_k, kv_v  [L, B, Hkv, >=max(ctx_len), hd] cached rotated keys / values (None if all
                ctx_len are 0)
    ctx_len     [B] committed tokens per sequence; row t sits at position ctx_len + depth(t)
    hidden_in   [B, k, d], or None on the first stage where rows are E[tokens]
    parent      draft tree (None = chain)
    Row t attends to every cached slot j < ctx_len and to drafted row s iff s is t or an
    ancestor of t.
    """
    m = model
    if hidden_in is not None:
        x = widen(hidden_in).copy()
    else:
        E = widen(get_weight("embed"))
        x = E[np.asarray(tokens, dtype=np.int64)]
    B, k, d = x.shape
    if parent is None:
        parent = list(range(k))
    A = ancestor_matrix(parent)
    depth = node_depths(parent)
    G = m.Hq // m.Hkv
    new_k = np.zeros((m.L, B, m.Hkv, k, m.hd), dtype=F64)
    new_v = np.zeros_like(new_k)
    taps: Dict[str, np.ndarray] = {}

    for l in range(m.L):
        p = f"l{l}."
        a = rms_norm(x, widen(get_weight(p + "g1")), m.eps)
        q = (a @ widen(get_weight(p + "wq")).T).reshape(B, k, m.Hq, m.hd)
        kk = (a @ widen(get_weight(p + "wk")).T).reshape(B, k, m.Hkv, m.hd)
        vv = (a @ widen(get_weight(p + "wv")).T).reshape(B, k, m.Hkv, m.hd)
        o = np.zeros((B, k, m.Hq, m.hd), dtype=F64)
        for b in range(B):
            C = int(ctx_len[b])
            pos = C + depth
            qb = rope(q[b], pos, m.rope_theta)                   # [k, Hq, hd]
            kb = rope(kk[b], pos, m.rope_theta)                  # [k, Hkv, hd]
            vb = vv[b]
            new_k[l, b] = kb.transpose(1, 0, 2)
            new_v[l, b] = vb.transpose(1, 0, 2)
            vis = np.concatenate([np.ones((k, C), dtype=bool), A], axis=1)
            for g in range(m.Hkv):
                if C > 0:
                    keys = np.concatenate([widen(kv_k[l, b, g, :C]), kb[:, g, :]], axis=0)
                    vals = np.concatenate([widen(kv_v[l, b, g, :C]), vb[:, g, :]], axis=0)
                else:
                    keys, vals = kb[:, g, :], vb[:, g, :]
                for h in range(g * G, (g + 1) * G):          # the query heads sharing kv head g
                    s = (qb[:, h, :] @ keys.T) / np.sqrt(F64(m.hd))   # [k, C + k]
                    s = np.where(vis, s, -np.inf)
                    s = s - s.max(axis=1, keepdims=True)
                    w = np.exp(s)
                    w = w / w.sum(axis=1, keepdims=True)
                    o[b, :, h, :] = w @ vals
        if want_taps:
            taps[p + "attn"] = o.reshape(B, k, m.Hq * m.hd).copy()
        x = x + o.reshape(B, k, m.Hq * m.hd) @ widen(get_weight(p + "wo")).T
        if want_taps:
            taps[p + "x_mid"] = x.copy()
        bn = rms_norm(x, widen(get_weight(p + "g2")), m.eps)
        gate = bn @ widen(get_weight(p + "wg")).T
        up = bn @ widen(get_weight(p + "wu")).T
        x = x + (silu(gate) * up) @ widen(get_weight(p + "wd")).T
        if want_taps:
            taps[p + "x_out"] = x.copy()

    logits = None
    if m.has_head:
        logits = rms_norm(x, widen(get_weight("gf")), m.eps) @ widen(get_weight("lm")).T
    return StageOut(hidden=x, logits=logits, new_k=new_k, new_v=new_v, taps=taps)


def kv_commit(kv_k: np.ndarray, kv_v: np.ndarray, ctx_len: np.ndarray, new_k: np.ndarray,
              new_v: np.ndarray, accepted_path: np.ndarray) -> np.ndarray:
    """Advance every sequence by its accepted drafted tokens (the paper's update
    x_{1:i+k} = x_{1:i} (+) y_{i+1:i+k}, section 2.1): the K/V rows of the accepted path's
    nodes, in path order, become slots ctx_len .. ctx_len + a - 1.  accepted_path [B, k]
    holds node ids 1..k, padded with -1.  Caches are modified in place; returns new lengths."""
    out = np.array(ctx_len, dtype=np.int64).copy()
    for b in range(accepted_path.shape[0]):
        a = 0
        for node in accepted_path[b]:
            if node < 0:
                break
            kv_k[:, b, :, out[b] + a, :] = new_k[:, b, :, node - 1, :]
            kv_v[:, b, :, out[b] + a, :] = new_v[:, b, :, node - 1, :]
            a += 1
        out[b] += a
    return out


# =============================================================================== accept
TREE_LONGEST = 0
TREE_FIRST_ACCEPTED = 1
TREE_LOSSLESS = 2      # recursive rejection over siblings drawn without replacement (see accept_lossless)


# Readings of the two loosely specified ingredients of the key rule (section 2.3):
NM_TOP_M = 0       # NormMatch = share of the top-M ids of P_t found in the top-M ids of q (the paper's example)
NM_OVERLAP = 1     # NormMatch = sum_v min(P_t(v), q(v)) = 1 - total variation distance of the two rows
H_TOKEN = 0        # H_m = -ln P_m(y): cross entropy of the drafted token under model m
H_ROW = 1          # H_m = -sum_v P_m(v) ln P_m(v): Shannon entropy of model m's row


@dataclass
class AcceptParams:
    lambda1: float = np.inf       # key if H_d > lambda1 * H_t
    lambda2: float = np.inf       # key if |P_t(y) - P_d(y)| > lambda2
    lambda3: float = -np.inf      # key if NormMatch < lambda3
    tau: float = 0.0              # relaxation for non-key tokens; 0 = the strict rule
    top_m: int = 8                # support size of NormMatch
    temperature: float = 1.0
    tree_mode: int = TREE_LONGEST
    norm_match_kind: int = 0      # NM_TOP_M or NM_OVERLAP
    entropy_kind: int = 0         # H_TOKEN or H_ROW


@dataclass
class AcceptOut:
    accepted_len: np.ndarray      # [B]
    next_token: np.ndarray        # [B]
    accepted_path: np.ndarray     # [B, k] node ids, -1 padded
    key: np.ndarray               # [B, k] bool
    node_accept: np.ndarray       # [B, k] bool, each node's own test
    tau_used: np.ndarray          # [B, k]
    ratio: np.ndarray             # [B, k]  P~(y)/q(y)  (inf when q(y) = 0 < P~(y))
    norm_match: np.ndarray        # [B, k]
    near_tie: np.ndarray          # [B] bit 0: accept test, bit 1: key rule, bit 2: resample draw (any node)
    tie_accept: np.ndarray        # [B, k] bool: node i's ratio P~(y)/q(y) lies within TIE_RATIO of its uniform
    tie_key: np.ndarray           # [B, k] bool: one of node i's key comparisons lies within its band (see accept)
    tie_draw: np.ndarray          # [B] bool: u_0 * S lies within TIE_CDF * S of a boundary of the cumulative sum


# Near-tie bands.  A decision is a comparison of two real numbers; an implementation that evaluates
# them in another precision or order may legitimately land on the other side when they are this
# close.  The oracle only REPORTS where that is the case (per node and per kind of decision); what a
# comparison of two implementations does with the flags is the test's business.
TIE_RATIO = 1e-3      # |P~(y)/q(y) - u_i|: the exception the acceptance test is allowed
TIE_LAMBDA = 1e-3     # relative distance of H_d from lambda1*H_t, of |P_t(y)-q(y)| from lambda2
TIE_TOP_M = 1e-5      # relative gap between the M-th and (M+1)-th largest entry of a row (top-M NormMatch)
TIE_OVERLAP = 1e-6    # absolute distance of the overlap NormMatch from lambda3
TIE_CDF = 1e-6        # distance of u_0*S from a cumulative-sum boundary, relative to S


def _new_out(B: int, k: int) -> AcceptOut:
    return AcceptOut(
        accepted_len=np.zeros(B, dtype=np.int32), next_token=np.zeros(B, dtype=np.int32),
        accepted_path=-np.ones((B, max(k, 1)), dtype=np.int32), key=np.zeros((B, k), dtype=bool),
        node_accept=np.zeros((B, k), dtype=bool), tau_used=np.zeros((B, k)), ratio=np.zeros((B, k)),
        norm_match=np.zeros((B, k)), near_tie=np.zeros(B, dtype=np.int32),
        tie_accept=np.zeros((B, k), dtype=bool), tie_key=np.zeros((B, k), dtype=bool),
        tie_draw=np.zeros(B, dtype=bool))


def _forced(force: Optional[np.ndarray], b: int, i: int, computed: bool) -> bool:
    """A decision as computed, unless the caller pins it (force[b, i-1] in {0, 1}; -1 = not pinned).
    Used by tests to ask what follows from a near-tie decision falling the other way."""
    if force is not None and int(force[b, i - 1]) >= 0:
        return bool(int(force[b, i - 1]))
    return computed


def _row_nm_and_tie(pt: np.ndarray, q: np.ndarray, prm: "AcceptParams"):
    """NormMatch of a row pair and whether it sits within its band of changing."""
    nm = row_norm_match(pt, q, prm)
    tie = False
    V = pt.shape[0]
    if prm.norm_match_kind == NM_TOP_M:
        for row in (pt, q):
            srt = np.sort(row)[::-1]
            if prm.top_m < V and srt[prm.top_m - 1] - srt[prm.top_m] < TIE_TOP_M * srt[prm.top_m - 1]:
                tie = True
    elif np.isfinite(prm.lambda3) and abs(nm - prm.lambda3) < TIE_OVERLAP:
        tie = True
    return nm, tie


def _key_tie(pt_y: float, q_y: float, h_t: float, h_d: float, prm: "AcceptParams") -> bool:
    """Whether the first or the second key criterion of a node lies within TIE_LAMBDA of its threshold."""
    tie = False
    with np.errstate(divide="ignore", invalid="ignore"):
        if np.isfinite(prm.lambda1) and np.isfinite(h_t) and np.isfinite(h_d) and \
                abs(h_d - prm.lambda1 * h_t) < TIE_LAMBDA * abs(prm.lambda1 * h_t):
            tie = True
    if np.isfinite(prm.lambda2) and abs(abs(pt_y - q_y) - prm.lambda2) < TIE_LAMBDA * prm.lambda2:
        tie = True
    return tie


def softmax_row(logits_row: np.ndarray, temperature: float) -> np.ndarray:
    z = logits_row.astype(F64) / F64(temperature)
    z = z - z.max()
    e = np.exp(z)
    return e / e.sum()


def top_m_ids(p: np.ndarray, M: int) -> np.ndarray:
    """Ids of the M largest entries; equal values go to the lower id."""
    order = np.lexsort((np.arange(p.shape[0]), -p))
    return order[:M]


def norm_match(pt: np.ndarray, q: np.ndarray, M: int) -> float:
    """Share of the top-M support of the target row found in the top-M support of the draft
    row (the paper's own example of NormMatch, section 2.3)."""
    return len(set(top_m_ids(pt, M).tolist()) & set(top_m_ids(q, M).tolist())) / float(M)


def norm_match_overlap(pt: np.ndarray, q: np.ndarray) -> float:
    """sum_v min(P_t(v), q(v)): the mass the two rows share (1 - total variation distance)."""
    return float(np.minimum(pt, q).sum())


def row_entropy(p: np.ndarray) -> float:
    """Shannon entropy -sum_v p(v) ln p(v) in nats, 0 ln 0 = 0."""
    nz = p[p > 0]
    return float(-(nz * np.log(nz)).sum())


def row_norm_match(pt: np.ndarray, q: np.ndarray, prm: "AcceptParams") -> float:
    return norm_match_overlap(pt, q) if prm.norm_match_kind == NM_OVERLAP else norm_match(pt, q, prm.top_m)


def key_entropies(pt: np.ndarray, q: np.ndarray, y: int, prm: "AcceptParams"):
    """(H_t, H_d) of the first key criterion under the chosen reading."""
    if prm.entropy_kind == H_ROW:
        return row_entropy(pt), row_entropy(q)
    with np.errstate(divide="ignore", invalid="ignore"):
        return float(-np.log(F64(pt[y]))), float(-np.log(F64(q[y])))


def is_key(pt_y: float, q_y: float, nm: float, prm: AcceptParams, h=None) -> bool:
    """Eq. "Key": any one of the three criteria makes the token a key token.  H_m is by default the
    cross entropy of the drafted token under model m, -ln P_m(y) (h = (H_t, H_d) overrides it, see
    key_entropies); the first criterion is used in product form so that H_t = 0 needs no division."""
    with np.errstate(divide="ignore", invalid="ignore"):
        if h is None:
            h_t = -np.log(F64(pt_y))
            h_d = -np.log(F64(q_y))
        else:
            h_t, h_d = F64(h[0]), F64(h[1])
        c1 = bool(h_d > prm.lambda1 * h_t)
    c2 = bool(abs(pt_y - q_y) > prm.lambda2)
    c3 = bool(nm < prm.lambda3)
    return c1 or c2 or c3


def softened_target(pt: np.ndarray, q: np.ndarray, tau: float) -> np.ndarray:
    """P~(v) = P_t(v)^(1-tau) q(v)^tau, renormalised; x^0 = 1 for every x including 0."""
    if tau == 0.0:
        return pt
    with np.errstate(divide="ignore", invalid="ignore"):
        w = np.power(pt, 1.0 - tau) * np.power(q, tau)
    return w / w.sum()


def inverse_cdf(weights: np.ndarray, u: float):
    """Smallest id v with sum_{j<=v} w_j > u * sum(w); if rounding leaves none, the largest id
    with positive weight.  Also returns how close u*S came to a boundary, relative to S."""
    c = np.cumsum(weights)
    S = c[-1]
    t = F64(u) * S
    v = int(np.searchsorted(c, t, side="right"))
    if v >= weights.shape[0]:
        v = int(np.nonzero(weights > 0)[0][-1])
    gap = np.min(np.abs(c - t)) / S if S > 0 else 0.0
    return v, float(gap)


def accept(logits: np.ndarray, draft_probs: np.ndarray, draft_tokens: np.ndarray,
           parent: Optional[Sequence[int]], uniforms: np.ndarray, prm: AcceptParams,
           tau_override: Optional[np.ndarray] = None, force_key: Optional[np.ndarray] = None,
           force_accept: Optional[np.ndarray] = None) -> AcceptOut:
    """Algorithm 1, lines 2-16, for B sequences.

    logits       [B, k+1, V]  row 0 follows the committed context, row i follows node i
    draft_probs  [B, k+1, V]  row p is the draft distribution node p's children were drawn from
    draft_tokens [B, k]       token of node i = 1..k
    parent       [k] in 0..k  (None = chain); parent[i-1] < i
    uniforms     [B, k+1]     u_i decides node i, u_0 draws the additional token
    tau_override [B, k]       if given, tau of node i regardless of the key rule
    force_key, force_accept [B, k] in {-1, 0, 1}: tests only -- pins the key flag / the outcome of
                 node i's own test (-1 = as computed), to follow a near-tie decision the other way
    """
    B, k1, V = logits.shape
    k = k1 - 1
    if parent is None:
        parent = list(range(k))
    parent = [int(p) for p in parent]
    if prm.temperature == 0.0:
        return accept_greedy(logits, draft_tokens, parent, prm)
    if prm.tree_mode == TREE_LOSSLESS:
        return accept_lossless(logits, draft_probs, draft_tokens, parent, uniforms, prm, force_key=force_key,
                               force_accept=force_accept)
    children: Dict[int, List[int]] = {}
    for i in range(1, k + 1):
        children.setdefault(parent[i - 1], []).append(i)
    depth = np.zeros(k + 1, dtype=np.int64)
    for i in range(1, k + 1):
        depth[i] = depth[parent[i - 1]] + 1

    out = _new_out(B, k)

    for b in range(B):
        pt_rows: Dict[int, np.ndarray] = {}
        nm_rows: Dict[int, tuple] = {}

        def target_row(p):
            if p not in pt_rows:
                pt_rows[p] = softmax_row(logits[b, p], prm.temperature)
            return pt_rows[p]

        ptilde_of: Dict[int, np.ndarray] = {}
        for i in range(1, k + 1):
            p = parent[i - 1]
            y = int(draft_tokens[b, i - 1])
            pt = target_row(p)
            q = draft_probs[b, p].astype(F64)
            if p not in nm_rows:
                nm_rows[p] = _row_nm_and_tie(pt, q, prm)
            nm, nm_tie = nm_rows[p]
            h_t, h_d = key_entropies(pt, q, y, prm)
            key = _forced(force_key, b, i, is_key(pt[y], q[y], nm, prm, (h_t, h_d)))
            out.tie_key[b, i - 1] = nm_tie or _key_tie(pt[y], q[y], h_t, h_d, prm)
            tau_i = 0.0 if key else prm.tau
            if tau_override is not None:
                tau_i = float(tau_override[b, i - 1])
            ptil = softened_target(pt, q, tau_i)
            ptilde_of[i] = ptil
            u = F64(uniforms[b, i])
            acc = _forced(force_accept, b, i, bool(u * q[y] < ptil[y]))
            with np.errstate(divide="ignore", invalid="ignore"):
                ratio = ptil[y] / q[y] if q[y] > 0 else (np.inf if ptil[y] > 0 else 0.0)
            out.tie_accept[b, i - 1] = abs(ratio - u) < TIE_RATIO
            out.key[b, i - 1] = key
            out.node_accept[b, i - 1] = acc
            out.tau_used[b, i - 1] = tau_i
            out.ratio[b, i - 1] = ratio
            out.norm_match[b, i - 1] = nm

        # which node ends the accepted path
        acc = out.node_accept[b]
        if prm.tree_mode == TREE_FIRST_ACCEPTED:
            v = 0
            while True:
                nxt = [c for c in children.get(v, []) if acc[c - 1]]
                if not nxt:
                    break
                v = nxt[0]
            vstar = v
        else:
            path_ok = np.zeros(k + 1, dtype=bool)
            path_ok[0] = True
            for i in range(1, k + 1):
                path_ok[i] = acc[i - 1] and path_ok[parent[i - 1]]
            vstar = 0
            for i in range(1, k + 1):
                if path_ok[i] and depth[i] > depth[vstar]:
                    vstar = i
        path = []
        n = vstar
        while n != 0:
            path.append(n)
            n = parent[n - 1]
        path.reverse()
        a = len(path)
        out.accepted_len[b] = a
        out.accepted_path[b, :a] = path

        # the additional token (Algorithm 1, line 16)
        u0 = F64(uniforms[b, 0])
        ch = children.get(vstar, [])
        if not ch:
            w = target_row(vstar)                 # whole window accepted: bonus from the target row
        else:
            ptil = ptilde_of[ch[0]]               # the softened target the rejected child was held to
            w = np.maximum(ptil - draft_probs[b, vstar].astype(F64), 0.0)
            if w.sum() == 0.0:
                w = ptil
        tok, gap = inverse_cdf(w, u0)
        out.tie_draw[b] = gap < TIE_CDF
        out.next_token[b] = tok
        out.near_tie[b] = (1 if out.tie_accept[b].any() else 0) | (2 if out.tie_key[b].any() else 0) | \
                          (4 if out.tie_draw[b] else 0)
    return out


def accept_lossless(logits: np.ndarray, draft_probs: np.ndarray, draft_tokens: np.ndarray, parent: Sequence[int],
                    uniforms: np.ndarray, prm: AcceptParams, force_key: Optional[np.ndarray] = None,
                    force_accept: Optional[np.ndarray] = None) -> AcceptOut:
    """Tree verification that keeps the target distribution when a node has several children.

    The paper verifies chains (section 2.1, Algorithm 1); for the token trees of the line of work
    it builds on (SpecInfer, cited in section 1) the accept test generalises to recursive rejection
    over the siblings, here for siblings drawn WITHOUT replacement from the parent's draft row:
    at node v with target row p_1 = P_t(. | v) and draft row q_1 = q_v, for the children c_1, c_2, ...
    in node order with tokens y_1, y_2, ...

        accept c_i  iff  u_{c_i} * q_i(y_i) < p_i(y_i)                     (probability min(1, p_i/q_i))
        on rejection    p_{i+1} = norm(max(0, p_i - q_i)),
                        q_{i+1} = q_i with y_i removed, renormalised        (the law of the next sibling)

    The first accepted child becomes v and the walk goes on with ITS rows; when every child of v is
    rejected (or v is a leaf) the additional token is drawn from the p that is left (the target row
    itself at a leaf) by inverse CDF with u_0.  The adaptive relaxation is not applied in this mode
    (tau_i = 0 for every node: the rule is about keeping P_t exactly); key flags and NormMatch are
    still reported.  node_accept and ratio are set for the nodes the walk tested, 0 elsewhere.
    A chain is the special case of one child per node and reproduces the strict chain rule."""
    B, k1, V = logits.shape
    k = k1 - 1
    children: Dict[int, List[int]] = {}
    for i in range(1, k + 1):
        children.setdefault(parent[i - 1], []).append(i)
    out = _new_out(B, k)
    for b in range(B):
        # key flags and NormMatch as in the other modes (reported only)
        for i in range(1, k + 1):
            p_row = parent[i - 1]
            y = int(draft_tokens[b, i - 1])
            pt = softmax_row(logits[b, p_row], prm.temperature)
            q = draft_probs[b, p_row].astype(F64)
            nm, nm_tie = _row_nm_and_tie(pt, q, prm)
            h_t, h_d = key_entropies(pt, q, y, prm)
            out.key[b, i - 1] = _forced(force_key, b, i, is_key(pt[y], q[y], nm, prm, (h_t, h_d)))
            out.norm_match[b, i - 1] = nm
            out.tie_key[b, i - 1] = nm_tie or _key_tie(pt[y], q[y], h_t, h_d, prm)
        v = 0
        path: List[int] = []
        while True:
            p = softmax_row(logits[b, v], prm.temperature)
            q = draft_probs[b, v].astype(F64).copy()
            taken = None
            for c in children.get(v, []):
                y = int(draft_tokens[b, c - 1])
                u = F64(uniforms[b, c])
                acc = _forced(force_accept, b, c, bool(u * q[y] < p[y]))
                with np.errstate(divide="ignore", invalid="ignore"):
                    ratio = p[y] / q[y] if q[y] > 0 else (np.inf if p[y] > 0 else 0.0)
                out.tie_accept[b, c - 1] = abs(ratio - u) < TIE_RATIO
                out.node_accept[b, c - 1] = acc
                out.ratio[b, c - 1] = ratio
                if acc:
                    taken = c
                    break
                r = np.maximum(p - q, 0.0)
                s = r.sum()
                if s > 0.0:
                    p = r / s
                q[y] = 0.0
                s = q.sum()
                if s > 0.0:
                    q = q / s
            if taken is None:
                break
            path.append(taken)
            v = taken
        a = len(path)
        out.accepted_len[b] = a
        out.accepted_path[b, :a] = path
        tok, gap = inverse_cdf(p, F64(uniforms[b, 0]))
        out.tie_draw[b] = gap < TIE_CDF
        out.next_token[b] = tok
        out.near_tie[b] = (1 if out.tie_accept[b].any() else 0) | (2 if out.tie_key[b].any() else 0) | \
                          (4 if out.tie_draw[b] else 0)
    return out


def accept_greedy(logits: np.ndarray, draft_tokens: np.ndarray, parent: Sequence[int], prm: AcceptParams) -> AcceptOut:
    """Verification at temperature 0 (the t = 0.0 rows of Table 1): the target is the one-hot
    distribution on arg max logits (ties to the lower id), so node i passes iff its token is the arg max
    of its parent's row, whatever the draft probabilities and the uniforms, and the additional token
    is the arg max of the row of the path's last node (the limit of both the residual and the bonus
    rule).  The accepted path follows tree_mode as at T > 0 (the lossless rule coincides with the
    first-accepted descent here: at most one child of a node can hold the arg max).  No relaxation,
    no key flags; ratio is 1 for a pass and 0 otherwise."""
    B, k1, V = logits.shape
    k = k1 - 1
    children: Dict[int, List[int]] = {}
    depth = np.zeros(k + 1, dtype=np.int64)
    for i in range(1, k + 1):
        children.setdefault(parent[i - 1], []).append(i)
        depth[i] = depth[parent[i - 1]] + 1
    out = _new_out(B, k)
    for b in range(B):
        best = [int(np.argmax(logits[b, r])) for r in range(k + 1)]      # numpy: first of equal maxima
        acc = np.zeros(k + 1, dtype=bool)
        acc[0] = True
        for i in range(1, k + 1):
            acc[i] = int(draft_tokens[b, i - 1]) == best[parent[i - 1]]
            out.node_accept[b, i - 1] = acc[i]
            out.ratio[b, i - 1] = 1.0 if acc[i] else 0.0
        if prm.tree_mode == TREE_LONGEST:
            ok = np.zeros(k + 1, dtype=bool)
            ok[0] = True
            vstar = 0
            for i in range(1, k + 1):
                ok[i] = acc[i] and ok[parent[i - 1]]
                if ok[i] and depth[i] > depth[vstar]:
                    vstar = i
        else:
            vstar = 0
            while True:
                nxt = [c for c in children.get(vstar, []) if acc[c]]
                if not nxt:
                    break
                vstar = nxt[0]
        path = []
        n = vstar
        while n != 0:
            path.append(n)
            n = parent[n - 1]
        path.reverse()
        out.accepted_len[b] = len(path)
        out.accepted_path[b, :len(path)] = path
        out.next_token[b] = best[vstar]
    return out
