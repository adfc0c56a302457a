"""GPU: a speculative decode loop over many rounds through the C ABI (section 2.1: draft k tokens,
verify them in one pass, accept, append, repeat), on a whole small bf16 model in one stage
(embedding + layers + head).  The draft is synthetic: the target itself, run one token at a time,
plus Gaussian logit noise.  Every round's accept decisions are checked against the oracle on the
logits the GPU produced; after the last round the cache rows that the commits left behind are
checked against an oracle forward pass over the emitted tokens, which pins stage + accept + commit
as they work together over ragged, advancing sequences.  Prints the average accepted length per
round (the "Avg len" column of Table 1 counts the same thing)."""
import numpy as np
import pytest
import torch

from oracle import dsd_oracle as O
from paper_2511_11733_amd import workloads as W
from tests import helpers as H
from tests.test_gpu_bf16 import mini

pytestmark = pytest.mark.gpu


def softmax64(z):
    z = z.astype(np.float64)
    z = z - z.max(-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(-1, keepdims=True)


@pytest.mark.parametrize("tau,noise", [(0.0, 0.5), (0.2, 1.0)])
def test_decode_loop_rounds(tau, noise):
    B, k, rounds = 3, 4, 8
    lens0 = [20, 33, 47]
    cfg, m, w, K, V, _, _, _ = mini(f"loop_tau{tau}", B=B, k=k, lens=lens0, head=True, V=4112, embed=True)
    rng = W.rng_for(cfg.seed, W.STREAM_DRAFT, f"loop{tau}")
    st = H.GpuStage(m, w, B, max(lens0) + rounds * (k + 1) + k + 2)
    st.import_kv(K, V, lens0)
    lens = np.array(lens0)
    pending = rng.integers(0, m.V, size=B).astype(np.int32)
    emitted = [[] for _ in range(B)]            # tokens whose K/V rows are committed behind the prompt
    prm = dict(tau=tau, lambda1=1.02, lambda2=1e-3, lambda3=0.3, top_m=8)
    acc_total = 0
    for r in range(rounds):
        # --- draft: the target one token at a time (rows land in the slots behind the committed ones)
        toks = np.zeros((B, k), dtype=np.int32)
        q = np.full((B, k + 1, m.V), 1.0 / m.V, dtype=np.float32)
        last = pending.copy()
        for i in range(k):
            st.kv.set_len((lens + i).tolist())
            _, lg = st.verify(tokens=last[:, None], want_hidden=False)
            z = lg.cpu().numpy()[:, 0].astype(np.float64) + noise * rng.standard_normal((B, m.V))
            qi = softmax64(z).astype(np.float32)
            q[:, i] = qi
            for b in range(B):
                toks[b, i] = W.draw_categorical(qi[b], float(rng.random()))
            last = toks[:, i].copy()
        st.kv.set_len(lens.tolist())
        # --- verify the pending token and the k drafted ones in one pass
        rows = np.concatenate([pending[:, None], toks], axis=1)
        _, lg = st.verify(tokens=rows, want_hidden=False)                 # [B, k+1, V]: row i follows node i
        u = rng.random((B, k + 1)).astype(np.float32)
        lg_np = lg.cpu().numpy()
        ora = O.accept(lg_np.astype(np.float64), q.astype(np.float64), toks, None, u, H.oracle_prm(O, prm))
        g = H.gpu_accept(st.ctx, lg, torch.from_numpy(q).to("cuda:0"), toks, None, u, prm)
        H.compare_accept(g, ora, f"round {r}", H.AcceptInputs(O, lg_np, q, toks, None, u, prm))
        a = ora.accepted_len.astype(np.int64)     # go on from the oracle's decisions (identical unless a near tie)
        # --- commit the pending token's row and the accepted ones (a chain: the first a+1 rows)
        n_rows = torch.from_numpy((a + 1).astype(np.int32)).to("cuda:0")
        H.D.dsd_kv_commit(st.ctx, st.kv, n_rows, None, B, k + 1)
        torch.cuda.synchronize()
        for b in range(B):
            emitted[b] += [int(pending[b])] + [int(t) for t in toks[b, :a[b]]]
        lens = lens + a + 1
        assert st.kv.get_len(B) == lens.tolist()
        pending = ora.next_token.astype(np.int32)
        acc_total += int(a.sum())
    avg = acc_total / (rounds * B)
    print(f"tau {tau}, noise {noise}: average accepted length {avg:.2f} of k = {k} over {rounds} rounds x {B} sequences")
    assert 0.3 < avg <= k
    # --- what the commits left in the cache == one oracle pass over the emitted tokens
    tol = H.TOL["bf16"]
    for b in range(B):
        n = len(emitted[b])
        assert n == lens[b] - lens0[b] and n <= 64
        Kb = np.concatenate([O.widen(K[:, b:b + 1, :, :lens0[b]]), np.zeros(K[:, b:b + 1, :, :1].shape[:3] + (n, K.shape[4]))], axis=3)
        Vb = np.concatenate([O.widen(V[:, b:b + 1, :, :lens0[b]]), np.zeros(V[:, b:b + 1, :, :1].shape[:3] + (n, V.shape[4]))], axis=3)
        ref = O.stage_forward(m, w.__getitem__, Kb, Vb, [lens0[b]], None, np.array([emitted[b]], dtype=np.int32))
        for l in range(m.L):
            gk, gv = st.new_rows(l, lens0[b], n, B)
            H.assert_close(gk[b:b + 1], ref.new_k[l], tol, f"committed K rows, layer {l}, sequence {b}")
            H.assert_close(gv[b:b + 1], ref.new_v[l], tol, f"committed V rows, layer {l}, sequence {b}")
