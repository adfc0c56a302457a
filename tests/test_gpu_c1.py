"""GPU parity, configuration 1: the tiny fp32 decoder (2 layers, d 256, 4/2 heads, head_dim 64,
FFN 688, vocab 4096), batch 1, 128 prior tokens prefilled, k = 4 chain, strict acceptance."""
import numpy as np
import pytest
import torch

from oracle import dsd_oracle as O
from paper_2511_11733_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c1():
    cfg = W.CONFIGS["c1"]
    m = cfg.model
    w = W.make_weights(m, cfg.seed)
    toks = W.make_prompt_tokens(cfg)                 # [1, 128]: 127 prefilled + 1 pending
    C = cfg.C
    pre = O.stage_forward(m, w.__getitem__, None, None, [0], None, toks[:, :C - 1])
    S = C + cfg.k + 8
    K = np.zeros((m.L, 1, m.Hkv, S, m.hd))
    V = np.zeros_like(K)
    K[:, :, :, :C - 1] = pre.new_k
    V[:, :, :, :C - 1] = pre.new_v
    # root row: feed the pending token
    root = O.stage_forward(m, w.__getitem__, K, V, [C - 1], None, toks[:, C - 1:C])
    lens = O.kv_commit(K, V, np.array([C - 1]), root.new_k, root.new_v, np.array([[1]], dtype=np.int32))
    assert lens[0] == C
    # sequential draft: q_i = softmax(target row i + noise), y_{i+1} ~ q_i
    noise = W.make_draft_noise(cfg, cfg.k + 1, m.V)
    ud = W.make_uniforms(cfg, cfg.k, tag="draft_draw", stream=W.STREAM_DRAFT)
    rows = [root.logits[0, 0]]
    qrows, draft = [], []
    for i in range(cfg.k):
        q = O.softmax_row(rows[i].astype(np.float32).astype(np.float64) + noise[0, i], 1.0)
        qrows.append(q)
        draft.append(W.draw_categorical(q, float(ud[0, i])))
        step = O.stage_forward(m, w.__getitem__, K, V, [C], None, np.array([draft]))
        rows.append(step.logits[0, i])
    qrows.append(O.softmax_row(rows[cfg.k] + noise[0, cfg.k], 1.0))
    full = O.stage_forward(m, w.__getitem__, K, V, [C], None, np.array([draft]))
    return dict(cfg=cfg, m=m, w=w, toks=toks, K=K, V=V, root=root, draft=np.array([draft], dtype=np.int32),
                full=full, q=np.stack(qrows)[None].astype(np.float32), S=S)


def test_c1_stage_verify_matches_oracle(c1):
    cfg, m = c1["cfg"], c1["m"]
    C, k = cfg.C, cfg.k
    st = H.GpuStage(m, c1["w"], 1, c1["S"])
    # the cache as it stood before the root call, then the root call on the GPU too
    st.import_kv(c1["K"][:, :, :, :C - 1], c1["V"][:, :, :, :C - 1], [C - 1])
    buf = torch.zeros((1, k + 1, m.V), dtype=torch.float32, device="cuda:0")
    st.verify(tokens=c1["toks"][:, C - 1:C], logits_buf=buf, logits_seq_stride=(k + 1) * m.V)
    alen = torch.ones(1, dtype=torch.int32, device="cuda:0")
    H.D.dsd_kv_commit(st.ctx, st.kv, alen, None, 1, 1)
    assert st.kv.get_len(1) == [C]
    hid, _ = st.verify(tokens=c1["draft"], logits_buf=buf, logits_offset=m.V, logits_seq_stride=(k + 1) * m.V)
    ref = np.concatenate([c1["root"].logits, c1["full"].logits], axis=1)
    nrms, worst = H.assert_close(H.to_np64(buf), ref, H.TOL["f32"], "c1 logits")
    print(f"c1 logits: normalised rms error {nrms:.2e}, worst/allowance {worst:.3f}")
    H.assert_close(H.to_np64(hid), c1["full"].hidden, H.TOL["f32"], "c1 hidden")
    for l in range(m.L):
        gk, gv = st.new_rows(l, C - 1, k + 1, 1)
        rk = np.concatenate([c1["root"].new_k[l], c1["full"].new_k[l]], axis=2)
        rv = np.concatenate([c1["root"].new_v[l], c1["full"].new_v[l]], axis=2)
        H.assert_close(gk, rk, H.TOL["f32"], f"c1 appended K layer {l}")
        H.assert_close(gv, rv, H.TOL["f32"], f"c1 appended V layer {l}")
    c1["gpu_logits"] = buf


def test_c1_accept_matches_oracle_both_ways(c1):
    cfg, m = c1["cfg"], c1["m"]
    k = cfg.k
    ctx = H.D.Context(0)
    u = W.make_uniforms(cfg, k + 1)
    prm = dict(tau=0.0)
    ref_logits = np.concatenate([c1["root"].logits, c1["full"].logits], axis=1).astype(np.float32)
    probs = torch.from_numpy(c1["q"]).to("cuda:0")
    cases = [("oracle logits", ref_logits)]
    if "gpu_logits" in c1:
        cases.append(("gpu logits", c1["gpu_logits"].cpu().numpy()))
    for name, lg in cases:
        # many uniform draws over the same rows: exercises accept, reject, resample and bonus
        for trial in range(24):
            uu = W.make_uniforms(cfg, k + 1, tag=f"u{trial}")
            if trial == 0:
                uu = u
            if trial == 1:
                uu[:, 1:] = 0.0          # everything accepted: bonus token
            ora = O.accept(lg.astype(np.float64), c1["q"].astype(np.float64), c1["draft"], None, uu,
                           H.oracle_prm(O, prm))
            g = H.gpu_accept(ctx, torch.from_numpy(lg).to("cuda:0"), probs, c1["draft"], None, uu, prm)
            H.compare_accept(g, ora, f"c1 accept ({name}, trial {trial})",
                             H.AcceptInputs(O, lg, c1["q"], c1["draft"], None, uu, prm))
            if trial == 1:
                assert ora.accepted_len[0] == k


def test_c1_commit_advances_cache(c1):
    cfg, m = c1["cfg"], c1["m"]
    C, k = cfg.C, cfg.k
    st = H.GpuStage(m, c1["w"], 1, c1["S"])
    st.import_kv(c1["K"][:, :, :, :C], c1["V"][:, :, :, :C], [C])
    st.verify(tokens=c1["draft"])
    alen = torch.tensor([3], dtype=torch.int32, device="cuda:0")
    path = torch.tensor([[1, 2, 3, -1]], dtype=torch.int32, device="cuda:0")
    H.D.dsd_kv_commit(st.ctx, st.kv, alen, path, 1, k)
    assert st.kv.get_len(1) == [C + 3]
    gk, gv = st.new_rows(0, C, 3, 1)
    H.assert_close(gk, c1["full"].new_k[0][:, :, :3], H.TOL["f32"], "committed K")
