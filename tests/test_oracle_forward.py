"""Pins for the oracle's stage forward (CPU only).

The paper prints no numeric example of the verification pass, so the forward is pinned to
(a) an independent library implementation of the same decoder architecture
    (transformers' Llama model, run in fp64 on random weights), and
(b) closed forms and invariants of the block.
"""
import numpy as np
import pytest
import torch

from oracle import dsd_oracle as O
from paper_2511_11733_amd import workloads as W

pytestmark = pytest.mark.filterwarnings("ignore")

# The library model builds its rotary cos/sin tables in float32 whatever the model dtype is,
# so agreement stops near 1e-6; any structural mistake (pairing, head mapping, mask, norm
# placement) shows up at O(0.1).
HF_ATOL = 2e-5


def tiny_model(L=3, d=64, Hq=4, Hkv=2, hd=16, F=112, V=97, head=True, embed=True, theta=1e4):
    return W.ModelCfg("t", L=L, d=d, Hq=Hq, Hkv=Hkv, hd=hd, F=F, V=V, dtype="f32", has_embed=embed,
                      has_head=head, rope_theta=theta)


def rand_weights(m, seed=0, std=0.3):
    """Larger spread than the workloads use, so that attention and the FFN matter."""
    rng = np.random.default_rng(seed)
    w = {}
    for name, shape, kind in W.weight_specs(m):
        if kind == "g":
            w[name] = 1.0 + 0.2 * rng.standard_normal(shape)
        else:
            w[name] = std * rng.standard_normal(shape) / np.sqrt(shape[-1] / 16.0)
    return w


# ------------------------------------------------------------------ (a) library model
def hf_llama(m, w):
    from transformers import LlamaConfig
    from transformers.models.llama.modeling_llama import LlamaForCausalLM

    cfg = LlamaConfig(vocab_size=m.V, hidden_size=m.d, intermediate_size=m.F, num_hidden_layers=m.L,
                      num_attention_heads=m.Hq, num_key_value_heads=m.Hkv, head_dim=m.hd,
                      rms_norm_eps=m.eps, rope_theta=m.rope_theta, attention_bias=False, mlp_bias=False,
                      tie_word_embeddings=False, max_position_embeddings=512,
                      attn_implementation="eager")
    net = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["gf"], "lm_head.weight": w["lm"]}
    names = {"g1": "input_layernorm.weight", "wq": "self_attn.q_proj.weight", "wk": "self_attn.k_proj.weight",
             "wv": "self_attn.v_proj.weight", "wo": "self_attn.o_proj.weight",
             "g2": "post_attention_layernorm.weight", "wg": "mlp.gate_proj.weight",
             "wu": "mlp.up_proj.weight", "wd": "mlp.down_proj.weight"}
    for l in range(m.L):
        for a, b in names.items():
            sd[f"model.layers.{l}.{b}"] = w[f"l{l}.{a}"]
    missing, unexpected = net.load_state_dict({k: torch.from_numpy(np.asarray(v, dtype=np.float64))
                                               for k, v in sd.items()}, strict=False)
    assert not [k for k in missing if "rotary" not in k and "inv_freq" not in k], missing
    assert not unexpected
    return net


@pytest.fixture(scope="module")
def hf_case():
    m = tiny_model()
    w = rand_weights(m)
    net = hf_llama(m, w)
    rng = np.random.default_rng(5)
    toks = rng.integers(0, m.V, size=(2, 21))
    with torch.no_grad():
        out = net(torch.from_numpy(toks), output_hidden_states=True, use_cache=False)
    return m, w, toks, out.logits.numpy(), [h.numpy() for h in out.hidden_states]


def test_prefill_matches_library_llama(hf_case):
    m, w, toks, logits, hs = hf_case
    r = O.stage_forward(m, w.__getitem__, None, None, [0, 0], None, toks)
    np.testing.assert_allclose(r.logits, logits, rtol=0, atol=HF_ATOL)


def test_cached_chain_matches_library_llama(hf_case):
    """Prefill 16 tokens, then verify a k=5 chain against the cache."""
    m, w, toks, logits, hs = hf_case
    P, k = 16, 5
    pre = O.stage_forward(m, w.__getitem__, None, None, [0, 0], None, toks[:, :P])
    kv_k = np.zeros((m.L, 2, m.Hkv, P + k, m.hd))
    kv_v = np.zeros_like(kv_k)
    kv_k[:, :, :, :P] = pre.new_k
    kv_v[:, :, :, :P] = pre.new_v
    r = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [P, P], None, toks[:, P:P + k])
    np.testing.assert_allclose(r.logits, logits[:, P:P + k], rtol=0, atol=HF_ATOL)


def test_stage_split_matches_library_hidden_states(hf_case):
    """A node hosts a contiguous block of layers: layers 0-1 without head give the library's
    hidden state after layer 2; layer 2 + head fed with it gives the library's logits."""
    m, w, toks, logits, hs = hf_case
    m_a = tiny_model(L=2, head=False)
    a = O.stage_forward(m_a, w.__getitem__, None, None, [0, 0], None, toks)
    np.testing.assert_allclose(a.hidden, hs[2], rtol=0, atol=HF_ATOL)
    m_b = tiny_model(L=1, embed=False)
    wb = {k.replace("l2.", "l0."): v for k, v in w.items() if k.startswith("l2.") or k in ("gf", "lm")}
    b = O.stage_forward(m_b, wb.__getitem__, None, None, [0, 0], a.hidden, None)
    np.testing.assert_allclose(b.logits, logits, rtol=0, atol=HF_ATOL)


def test_unequal_context_lengths_match_library(hf_case):
    m, w, toks, logits, hs = hf_case
    k = 3
    lens = [16, 11]
    kv_k = np.zeros((m.L, 2, m.Hkv, 24, m.hd))
    kv_v = np.zeros_like(kv_k)
    draft = np.zeros((2, k), dtype=np.int64)
    for b, P in enumerate(lens):
        pre = O.stage_forward(m, w.__getitem__, None, None, [0], None, toks[b:b + 1, :P])
        kv_k[:, b, :, :P] = pre.new_k[:, 0]
        kv_v[:, b, :, :P] = pre.new_v[:, 0]
        draft[b] = toks[b, P:P + k]
    r = O.stage_forward(m, w.__getitem__, kv_k, kv_v, lens, None, draft)
    for b, P in enumerate(lens):
        np.testing.assert_allclose(r.logits[b], logits[b, P:P + k], rtol=0, atol=HF_ATOL)


# ------------------------------------------------------------------ (b) closed forms
def test_rms_norm_softmax_silu_match_torch_routines():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 7, 40))
    g = 1 + 0.1 * rng.standard_normal(40)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (40,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(O.rms_norm(x, g, 1e-5), ref, atol=1e-13)
    np.testing.assert_allclose(O.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), atol=1e-14)
    np.testing.assert_allclose(O.softmax_row(x[0, 0], 0.7),
                               torch.softmax(torch.from_numpy(x[0, 0]) / 0.7, 0).numpy(), atol=1e-15)


def test_rope_closed_forms():
    rng = np.random.default_rng(1)
    v = rng.standard_normal((5, 3, 8))
    # position 0 is the identity
    np.testing.assert_allclose(O.rope(v, np.zeros(5), 1e4), v, atol=0)
    # rotations preserve norms
    r = O.rope(v, np.arange(5) + 100, 1e4)
    np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-13)
    # head_dim 2: a plain rotation of the pair by `pos` radians (frequency theta^0 = 1)
    p = np.array([[[1.0, 0.0]]])
    np.testing.assert_allclose(O.rope(p, np.array([0.5]), 1e4)[0, 0], [np.cos(0.5), np.sin(0.5)], atol=1e-15)
    # the second pair of head_dim 4 turns at theta^(-1/2)
    p = np.array([[[0.0, 1.0, 0.0, 0.0]]])
    out = O.rope(p, np.array([3.0]), 1e4)[0, 0]
    np.testing.assert_allclose(out, [0, np.cos(0.03), 0, np.sin(0.03)], atol=1e-15)
    # scores depend on the position difference only
    q = rng.standard_normal((1, 1, 8))
    kx = rng.standard_normal((1, 1, 8))
    s1 = O.rope(q, np.array([7]), 5e5)[0, 0] @ O.rope(kx, np.array([3]), 5e5)[0, 0]
    s2 = O.rope(q, np.array([1007]), 5e5)[0, 0] @ O.rope(kx, np.array([1003]), 5e5)[0, 0]
    assert abs(s1 - s2) < 1e-10


def small_stage(seed=0, B=2, C=9, k=4, **kw):
    m = tiny_model(L=2, head=False, embed=False, **kw)
    w = rand_weights(m, seed)
    rng = np.random.default_rng(seed + 1)
    kv_k = rng.standard_normal((m.L, B, m.Hkv, C + k, m.hd))
    kv_v = rng.standard_normal((m.L, B, m.Hkv, C + k, m.hd))
    h = rng.standard_normal((B, k, m.d))
    return m, w, kv_k, kv_v, h


def test_zero_output_projections_leave_hidden_unchanged():
    m, w, kv_k, kv_v, h = small_stage()
    for l in range(m.L):
        w[f"l{l}.wo"] = np.zeros_like(w[f"l{l}.wo"])
        w[f"l{l}.wd"] = np.zeros_like(w[f"l{l}.wd"])
    r = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [9, 9], h, None)
    np.testing.assert_array_equal(r.hidden, h)


def test_single_visible_key_returns_its_value_row():
    """k=1 with an empty cache: the row sees only itself, so attention returns its own V row."""
    m, w, kv_k, kv_v, h = small_stage(k=1, C=0)
    r = O.stage_forward(m, w.__getitem__, None, None, [0, 0], h, None, want_taps=True)
    G = m.Hq // m.Hkv
    attn = r.taps["l0.attn"].reshape(2, 1, m.Hq, m.hd)
    for hq in range(m.Hq):
        np.testing.assert_allclose(attn[:, 0, hq], r.new_v[0, :, hq // G, 0], atol=1e-14)


def test_attention_core_matches_torch_sdpa():
    """With identity-like projections removed from the picture: compare the attention tap with
    torch's scaled_dot_product_attention on the same rotated q, k, v."""
    m, w, kv_k, kv_v, h = small_stage(B=1, C=6, k=3)
    r = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [6], h, None, want_taps=True)
    a = O.rms_norm(h, w["l0.g1"], m.eps)
    q = (a @ w["l0.wq"].T).reshape(1, 3, m.Hq, m.hd)
    q = O.rope(q[0], np.arange(6, 9), m.rope_theta)                       # [k, Hq, hd]
    keys = np.concatenate([kv_k[0, 0, :, :6], r.new_k[0, 0]], axis=1)     # [Hkv, 9, hd]
    vals = np.concatenate([kv_v[0, 0, :, :6], r.new_v[0, 0]], axis=1)
    G = m.Hq // m.Hkv
    mask = torch.ones(3, 9, dtype=torch.bool)
    mask[:, 6:] = torch.tril(torch.ones(3, 3, dtype=torch.bool))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q.transpose(1, 0, 2))[None],
        torch.from_numpy(np.repeat(keys, G, axis=0))[None],
        torch.from_numpy(np.repeat(vals, G, axis=0))[None], attn_mask=mask)[0].numpy()   # [Hq, k, hd]
    np.testing.assert_allclose(r.taps["l0.attn"].reshape(3, m.Hq, m.hd), ref.transpose(1, 0, 2), atol=1e-12)


def test_chain_equals_successive_single_row_steps():
    """Causality: verifying k rows at once equals k one-row decode steps with commits between."""
    m, w, kv_k, kv_v, h = small_stage()
    B, k = h.shape[:2]
    r = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [9, 9], h, None)
    kk, kvv = kv_k.copy(), kv_v.copy()
    lens = np.array([9, 9])
    for t in range(k):
        s = O.stage_forward(m, w.__getitem__, kk, kvv, lens, h[:, t:t + 1], None)
        np.testing.assert_allclose(s.hidden[:, 0], r.hidden[:, t], atol=1e-12)
        lens = O.kv_commit(kk, kvv, lens, s.new_k, s.new_v, np.ones((B, 1), dtype=np.int32))
    assert lens.tolist() == [13, 13]
    np.testing.assert_allclose(kk[:, :, :, 9:13], r.new_k, atol=1e-12)


def test_batch_permutation_equivariance():
    m, w, kv_k, kv_v, h = small_stage(B=3)
    r = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [9, 5, 7], h, None)
    perm = [2, 0, 1]
    rp = O.stage_forward(m, w.__getitem__, kv_k[:, perm], kv_v[:, perm], [7, 9, 5], h[perm], None)
    np.testing.assert_allclose(rp.hidden, r.hidden[perm], atol=1e-13)


def test_tree_paths_equal_chains():
    """Every root-to-leaf path of a draft tree must come out as if it had been verified alone as
    a chain (ancestor mask + depth positions).  The degenerate one-child tree is the chain."""
    parent = W.ranked_tree_parents((3, 2, 2), 10)
    k = len(parent)
    m, w, kv_k, kv_v, h = small_stage(B=1, C=5, k=k)
    r = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [5], h, None, parent=parent)
    ch = W.children_of(parent)
    leaves = [i for i in range(1, k + 1) if i not in ch]
    assert len(leaves) >= 3
    for leaf in leaves:
        path = []
        n = leaf
        while n:
            path.append(n)
            n = int(parent[n - 1])
        path.reverse()
        idx = [p - 1 for p in path]
        c = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [5], h[:, idx], None)
        np.testing.assert_allclose(c.hidden[0], r.hidden[0, idx], atol=1e-12)
    chain = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [5], h, None, parent=list(range(k)))
    none = O.stage_forward(m, w.__getitem__, kv_k, kv_v, [5], h, None)
    np.testing.assert_array_equal(chain.hidden, none.hidden)


def test_ancestor_matrix_matches_bitmask_generator():
    parent = W.ranked_tree_parents()
    A = O.ancestor_matrix(parent)
    bits = W.tree_mask_bits(parent)
    for t in range(len(parent)):
        for s in range(len(parent)):
            assert bool(A[t, s]) == bool((int(bits[t]) >> s) & 1)
    assert O.node_depths(parent).tolist() == W.tree_depths(parent).tolist()
    with open(__file__.rsplit("/", 1)[0] + "/golden/tree_32_parents.txt") as f:
        gold = [int(x) for x in f.read().split("#")[0].split()]
    assert parent.tolist() == gold


def test_kv_commit_moves_accepted_path_rows():
    rng = np.random.default_rng(3)
    L, B, H, hd, C, k = 2, 2, 2, 4, 3, 4
    kk = rng.standard_normal((L, B, H, C + k, hd))
    vv = rng.standard_normal((L, B, H, C + k, hd))
    nk = rng.standard_normal((L, B, H, k, hd))
    nv = rng.standard_normal((L, B, H, k, hd))
    path = np.array([[2, 4, -1, -1], [-1, -1, -1, -1]], dtype=np.int32)
    k0 = kk.copy()
    lens = O.kv_commit(kk, vv, np.array([C, C]), nk, nv, path)
    assert lens.tolist() == [C + 2, C]
    np.testing.assert_array_equal(kk[:, 0, :, C], nk[:, 0, :, 1])
    np.testing.assert_array_equal(kk[:, 0, :, C + 1], nk[:, 0, :, 3])
    np.testing.assert_array_equal(vv[:, 0, :, C + 1], nv[:, 0, :, 3])
    np.testing.assert_array_equal(kk[:, 1], k0[:, 1])
