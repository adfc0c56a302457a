"""GPU parity of the bf16 verification pass against the fp64 oracle on reduced copies of the
benchmark workloads: same generators and value distributions, sizes the oracle finishes in
seconds, several tiles plus ragged tails in every dimension that is tiled (rows, context,
vocabulary), unequal context lengths, chain and tree masks."""
import os

import numpy as np
import pytest
import torch

from oracle import dsd_oracle as O
from paper_2511_11733_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def mini(name, B, k, lens, tree=None, head=False, L=2, d=512, Hq=8, Hkv=2, F=1536, V=8000, seed=3, embed=False):
    base = W.CONFIGS["c3" if head else "c2"]
    cfg = W.scaled(base, name=name, B=B, k=k, C=max(lens), seed=seed, L=L, d=d, Hq=Hq, Hkv=Hkv, F=F,
                   V=V if (head or embed) else 0, has_head=head, has_embed=embed)
    m = cfg.model
    w = W.make_weights(m, cfg.seed)
    K, Vv = W.make_kv(cfg)
    hid = W.make_hidden(cfg)
    parent = None
    if tree is not None:
        parent = W.ranked_tree_parents(*tree)
        assert len(parent) == k
    return cfg, m, w, K, Vv, hid, parent, list(lens)


def check(case, simple=False, no_tiled=False):
    cfg, m, w, K, V, hid, parent, lens = case
    ref = O.stage_forward(m, w.__getitem__, K, V, lens, hid, None, parent=parent)
    if simple:
        os.environ["DSD_PATH"] = "simple"
    if no_tiled:
        os.environ["DSD_NO_TILED"] = "1"
    try:
        st = H.GpuStage(m, w, cfg.B, max(lens) + cfg.k + 3)
    finally:
        os.environ.pop("DSD_PATH", None)
        os.environ.pop("DSD_NO_TILED", None)
    st.import_kv(K, V, lens)
    out, lg = st.verify(hidden=hid, parent=parent)
    tol = H.TOL["bf16"]
    nrms, worst = H.assert_close(H.to_np64(out), ref.hidden, tol, f"{cfg.name} hidden")
    print(f"{cfg.name}: hidden normalised rms error {nrms:.2e}, worst/allowance {worst:.3f}")
    if m.has_head:
        nrms, worst = H.assert_close(H.to_np64(lg), ref.logits, tol, f"{cfg.name} logits")
        print(f"{cfg.name}: logits normalised rms error {nrms:.2e}, worst/allowance {worst:.3f}")
    for l in range(m.L):
        for b in range(cfg.B):
            gk, gv = st.new_rows(l, lens[b], cfg.k, cfg.B)
            H.assert_close(gk[b], ref.new_k[l, b], tol, f"{cfg.name} appended K layer {l} seq {b}")
            H.assert_close(gv[b], ref.new_v[l, b], tol, f"{cfg.name} appended V layer {l} seq {b}")
    # the committed part of the cache is untouched
    if min(lens) > 0:
        gk, gv = st.new_rows(0, 0, min(lens), cfg.B)
        np.testing.assert_array_equal(gk, O.widen(K[0][:, :, :min(lens)]))
        np.testing.assert_array_equal(gv, O.widen(V[0][:, :, :min(lens)]))
    return st, ref


def test_mid_stage_chain_ragged_lengths():
    check(mini("mini_mid", B=3, k=5, lens=[300, 77, 130]))


def test_mid_stage_chain_generic_kernels():
    check(mini("mini_mid_generic", B=3, k=5, lens=[300, 77, 130]), simple=True)


def test_final_stage_tree():
    check(mini("mini_tree", B=2, k=10, lens=[129, 64], tree=((3, 2, 2), 10), head=True))


def test_more_rows_four_row_tiles():
    check(mini("mini_m64", B=8, k=8, lens=[200, 31, 64, 65, 1, 255, 256, 100], head=True, V=4112))


def test_max_rows_tree_32_nodes():
    check(mini("mini_m128", B=4, k=32, lens=[150, 90, 33, 64], tree=((4, 3, 2, 2, 1, 1), 32), head=True, L=1))


def test_long_chains_three_and_four_row_groups():
    """40 and 64 drafted rows per sequence: 160 and 256 query rows per kv head, i.e. five and eight waves of
    two row tiles sharing every run's staged K/V, and k at its limit."""
    check(mini("mini_k40", B=2, k=40, lens=[70, 129], head=True, V=4112, L=1))
    check(mini("mini_k64", B=2, k=64, lens=[33, 64], L=1))
    # 8 query heads per kv head and 40 drafted rows: 320 query rows per kv head, more than one attention launch
    # holds (256): the rows go through in two groups, 16 tiles and 4 tiles
    check(mini("mini_k40_g8", B=1, k=40, lens=[70], Hq=16, Hkv=2, d=1024, F=1536, L=1))


def test_shapes_the_panel_path_does_not_take():
    """An FFN width that is no multiple of 512 keeps the panel GEMMs out: the one-workgroup-per-tile
    kernels then carry any row count themselves (2, 4 and 8 row tiles here), as they did before the
    panel path existed.  Also: one query head per kv head, and a vocabulary of two column tiles."""
    check(mini("mini_f1792_m24", B=3, k=8, lens=[40, 9, 64], F=1792, L=1))
    check(mini("mini_f1792_m64", B=8, k=8, lens=[40, 9, 64, 1, 100, 33, 80, 17], F=1792, head=True, V=4112, L=1))
    check(mini("mini_f1792_m128", B=16, k=8, lens=[30 + 5 * b for b in range(16)], F=1792, L=1))
    check(mini("mini_mha", B=2, k=5, lens=[70, 33], Hq=4, Hkv=4, head=True, V=32, L=1))


def test_head_dim_64_in_bf16_takes_the_generic_kernels():
    lens = [50, 17]
    cfg = W.scaled(W.CONFIGS["c3"], name="mini_hd64", B=2, k=5, C=max(lens), seed=3, L=2, d=256, Hq=4, Hkv=2, hd=64,
                   F=512, V=1000, has_head=True, has_embed=False)
    m = cfg.model
    check((cfg, m, W.make_weights(m, cfg.seed), *W.make_kv(cfg), W.make_hidden(cfg), None, lens))


def test_both_gemm_paths_on_the_same_case():
    """2, 5, 10, 15 and 40 rows through the default path (the panel GEMMs) and, with DSD_NO_TILED,
    through the one-workgroup-per-tile kernels: each against the oracle."""
    for name, B, k in (("both_m2", 1, 2), ("both_m5", 1, 5), ("both_m10", 2, 5), ("both_m15", 3, 5), ("both_m40", 5, 8)):
        case = mini(name, B=B, k=k, lens=[90 + 13 * b for b in range(B)], head=True, V=4112, L=2)
        check(case)
        check(case, no_tiled=True)


def test_wide_ffn_with_many_rows():
    """A 70B-wide FFN at 80 and 128 rows: gate/up has a workgroup of 256 columns per compute unit, so it
    runs 8 computing waves with 6 and 8 row tiles."""
    check(mini("mini_wide80", B=10, k=8, lens=[20 + 3 * b for b in range(10)], F=28672, L=1))
    check(mini("mini_wide128", B=16, k=8, lens=[20 + 3 * b for b in range(16)], F=28672, L=1))


def test_large_vocabulary_head_with_many_rows():
    """From 65 rows on a vocabulary of at least 256 column blocks of 256 ids runs the LM head with 8
    computing waves per workgroup (6 and 8 row tiles): 80 and 128 rows, V = 66000."""
    check(mini("mini_v66k_m80", B=10, k=8, lens=[20 + 3 * b for b in range(10)], head=True, V=66000, L=1))
    check(mini("mini_v66k_m128", B=16, k=8, lens=[20 + 3 * b for b in range(16)], head=True, V=66000, L=1))


def test_few_rows_on_the_panel_path_for_wide_models():
    """A d_model of more than 16 tiles per compute unit (here 4608: 288 tiles on 256 CUs) takes the panel
    GEMMs at every row count: 1, 5 and 10 rows."""
    for B, k in ((1, 1), (1, 5), (2, 5)):
        check(mini(f"mini_d4608_m{B * k}", B=B, k=k, lens=[70, 33][:B], d=4608, Hq=36, Hkv=4, F=2048, L=1))


def test_two_and_three_row_tiles():
    check(mini("mini_m24", B=4, k=6, lens=[100, 5, 64, 33]))
    check(mini("mini_m40", B=5, k=8, lens=[17, 200, 63, 1, 128], head=True, V=4112, L=1))


def test_six_row_tiles():
    # 80 and 96 rows both run the 6-tile kernels (row tiles taken in two halves of 3)
    check(mini("mini_m80", B=10, k=8, lens=[30, 200, 64, 65, 1, 100, 7, 150, 90, 129], head=True, V=4112, L=1))
    check(mini("mini_m96", B=12, k=8, lens=[60] * 12, L=1))


def test_wide_ffn_picks_eight_computing_waves():
    # with this many gate/up columns the GEMM for up to 64 rows runs 8 computing waves per workgroup
    check(mini("mini_wide24", B=4, k=6, lens=[50, 20, 64, 9], F=26624, L=1))
    check(mini("mini_wide64", B=8, k=8, lens=[50, 20, 64, 9, 1, 100, 33, 80], F=26624, L=1))


def test_first_node_block_with_embedding():
    """A block that starts the pipeline: rows come from the embedding table (ids out of range are
    clamped), here with the head as well, i.e. a whole small model in one call."""
    for name, B, k in (("mini_embed5", 1, 5), ("mini_embed40", 5, 8)):
        cfg, m, w, K, V, hid, parent, lens = mini(name, B=B, k=k, lens=[33 + 20 * b for b in range(B)], head=True,
                                                  V=4112, embed=True)
        toks = W.rng_for(cfg.seed, W.STREAM_STATE, "ids").integers(0, m.V, size=(B, k), dtype=np.int32)
        ref = O.stage_forward(m, w.__getitem__, K, V, lens, None, toks)
        st = H.GpuStage(m, w, cfg.B, max(lens) + cfg.k + 3)
        st.import_kv(K, V, lens)
        out, lg = st.verify(tokens=toks)
        tol = H.TOL["bf16"]
        H.assert_close(H.to_np64(out), ref.hidden, tol, f"{name} hidden")
        nrms, worst = H.assert_close(H.to_np64(lg), ref.logits, tol, f"{name} logits")
        print(f"{name}: logits normalised rms error {nrms:.2e}, worst/allowance {worst:.3f}")


def test_empty_context():
    check(mini("mini_empty", B=2, k=6, lens=[0, 0]))


def test_long_context_is_cut_into_hundreds_of_key_runs():
    """One sequence with 20 000 cached positions and two kv heads: the attention takes the most runs per
    (sequence, head) that runs of 64 keys allow (about 300), and the combine kernel merges them all."""
    check(mini("mini_long", B=1, k=5, lens=[20000], L=1))


def test_many_sequences_ragged_lengths():
    """40 sequences x 8 kv heads = 320 (sequence, head) units, more than one per compute unit: few runs per
    unit, and lengths from empty to several runs long in the same launch."""
    lens = [(37 * b) % 700 for b in range(40)]
    check(mini("mini_b40", B=40, k=3, lens=lens, Hq=8, Hkv=8, L=1))


def test_k1_plain_decode_step():
    check(mini("mini_k1", B=5, k=1, lens=[40, 41, 63, 64, 65]))


def test_wide_gqa_group_70b_like():
    # 8 query heads per kv head as in the 70B-shaped workload: 6*8 = 48 query rows per kv head
    check(mini("mini_70b", B=2, k=6, lens=[140, 200], Hq=16, Hkv=2, d=1024, F=2048))


# ---- d_model 2048 (K a multiple of 2048), few rows at a narrower model
def test_d2048_mid_stage_chain():
    check(mini("d2048_mid", B=1, k=5, lens=[300], d=2048, Hq=16, Hkv=4, F=4096))
    check(mini("d2048_mid8", B=2, k=4, lens=[77, 130], d=2048, Hq=16, Hkv=4, F=4096))


def test_d2048_final_stage_tree():
    check(mini("d2048_tree", B=1, k=10, lens=[129], tree=((3, 2, 2), 10), head=True, d=2048, Hq=16, Hkv=4,
               F=4096, V=4112))
    check(mini("d2048_tree8", B=1, k=8, lens=[129], tree=((3, 2, 2), 8), head=True, d=2048, Hq=16, Hkv=4,
               F=4096, V=4112))


def test_d2048_empty_context_and_k1():
    check(mini("d2048_empty", B=1, k=6, lens=[0], d=2048, Hq=16, Hkv=4, F=4096, L=1))
    check(mini("d2048_k1", B=5, k=1, lens=[40, 41, 63, 64, 65], d=2048, Hq=16, Hkv=4, F=4096, L=3))


def test_d2048_one_kv_head_pair():
    case = mini("d2048_gqa8", B=1, k=8, lens=[200], d=2048, Hq=16, Hkv=2, F=6144, head=True, V=4096)
    check(case)


def wide_ffn_case(name, B, k, spread):
    """A block whose FFN intermediates SiLU(gate)*up are large: gate and up rows of spread `spread` (weights
    N(0, (spread/sqrt(d))^2)), a down projection small enough to bring the result back to the size of the
    residual stream.  The matrix-core path carries those intermediates as fp16 operands (limit 65504)."""
    case = mini(name, B=B, k=k, lens=[40 + 7 * b for b in range(B)], L=2, d=512, F=1024)
    cfg, m, w, K, V, hid, parent, lens = case
    rng = np.random.default_rng(5)
    for l in range(m.L):
        for nm in ("wg", "wu"):
            w[f"l{l}.{nm}"] = W.f32_to_bf16_bits((rng.standard_normal((m.F, m.d)) * spread / np.sqrt(m.d)).astype(np.float32))
        w[f"l{l}.wd"] = W.f32_to_bf16_bits((rng.standard_normal((m.d, m.F)) / (spread * spread * np.sqrt(m.F))).astype(np.float32))
    return case


def stage_on_path(m, w, B, slots, no_tiled):
    """A stage on a context of its own; no_tiled: the one-workgroup-per-tile GEMMs at every row count."""
    if no_tiled:
        os.environ["DSD_NO_TILED"] = "1"
    try:
        return H.GpuStage(m, w, B, slots)
    finally:
        os.environ.pop("DSD_NO_TILED", None)


# both GEMM paths, and the panel path with two row-tile counts
BOTH_PATHS = [(1, 5, False), (4, 6, False), (1, 5, True)]


@pytest.mark.parametrize("B,k,no_tiled", BOTH_PATHS)
def test_large_ffn_intermediates_inside_the_fp16_range_keep_parity(B, k, no_tiled):
    """SiLU(gate)*up up to about 3e4: inside the range, so parity with the oracle holds and nothing is counted."""
    case = wide_ffn_case(f"ffn_big_{B * k}", B, k, spread=40.0)
    cfg, m, w, K, V, hid, parent, lens = case
    ref = O.stage_forward(m, w.__getitem__, K, V, lens, hid, None, want_taps=False)
    st = stage_on_path(m, w, cfg.B, max(lens) + cfg.k + 3, no_tiled)
    st.import_kv(K, V, lens)
    out, _ = st.verify(hidden=hid)
    H.assert_close(H.to_np64(out), ref.hidden, H.TOL["bf16"], f"{cfg.name} hidden")
    assert st.ctx.stage_status() == 0


@pytest.mark.parametrize("B,k,no_tiled", BOTH_PATHS)
def test_ffn_intermediates_beyond_the_fp16_range_are_reported(B, k, no_tiled):
    """SiLU(gate)*up in the 1e6 range: the fp16 operands saturate, the result is not the model's, and
    dsd_stage_status says so (and is clean again afterwards)."""
    case = wide_ffn_case(f"ffn_over_{B * k}", B, k, spread=400.0)
    cfg, m, w, K, V, hid, parent, lens = case
    bn = O.rms_norm(O.widen(hid), O.widen(w["l0.g2"]), m.eps)       # the order of magnitude, from the oracle's pieces
    hmax = np.abs(O.silu(bn @ O.widen(w["l0.wg"]).T) * (bn @ O.widen(w["l0.wu"]).T)).max()
    assert hmax > 2 * 65504
    st = stage_on_path(m, w, cfg.B, max(lens) + cfg.k + 3, no_tiled)
    st.import_kv(K, V, lens)
    st.verify(hidden=hid)
    with pytest.raises(H.D.DsdError, match="65504"):
        st.ctx.stage_status()
    assert st.ctx.stage_status() == 0                               # the count was cleared by the failing check
    # an ordinary block on the same context afterwards: clean
    cfg2, m2, w2, K2, V2, hid2, parent2, lens2 = mini("after_overflow", B=B, k=k, lens=[33] * B)
    st2 = H.GpuStage(m2, w2, B, 33 + k + 3, ctx=st.ctx)
    st2.import_kv(K2, V2, lens2)
    st2.verify(hidden=hid2)
    assert st.ctx.stage_status() == 0


def test_shape_errors():
    case = mini("mini_err", B=2, k=4, lens=[10, 10])
    cfg, m, w, K, V, hid, parent, lens = case
    st = H.GpuStage(m, w, 2, 16)
    st.import_kv(K, V, lens)
    with pytest.raises(H.D.DsdError):            # 13 + 4 rows exceed 16 slots
        st.kv.set_len([13, 10])
        st.verify(hidden=hid)
    st.kv.set_len(lens)
    with pytest.raises(H.D.DsdError):            # logits from a block without head
        lg = torch.zeros((2, 4, 8), dtype=torch.float32, device="cuda:0")
        H.D.dsd_stage_verify(st.ctx, st.w, st.kv, st._cast(hid), None, None, None, 2, 4, None, lg)
    with pytest.raises(H.D.DsdError):            # batch larger than the cache
        H.D.dsd_stage_verify(st.ctx, st.w, st.kv, st._cast(hid), None, None, None, 3, 4, st._cast(hid), None)


def test_stage_replays_from_a_hip_graph():
    """Once the workspace has its size the call issues only kernels on the context's stream, so a caller
    may capture it; every replay (with eager work and synchronisations in between) must reproduce the
    eager result bit for bit: every sum on the path is taken in a fixed order (K slices of the GEMMs
    on the panel path land in buffers of their own and are added up slice by slice), so two runs
    on the same inputs may not differ at all."""
    for name, B, k in (("graph_m5", 1, 5), ("graph_m40", 5, 8)):
        cfg, m, w, K, V, hid, parent, lens = mini(name, B=B, k=k, lens=[70 + 9 * b for b in range(B)], head=True,
                                                  V=4112, L=2)
        stream = torch.cuda.Stream()
        ctx = H.D.Context(0, stream)
        st = H.GpuStage(m, w, cfg.B, max(lens) + cfg.k + 3, ctx=ctx)
        with torch.cuda.stream(stream):
            st.import_kv(K, V, lens)
            h = st._cast(hid)
            out = torch.empty((B, k, m.d), dtype=torch.bfloat16, device="cuda:0")
            lg = torch.empty((B, k, m.V), dtype=torch.float32, device="cuda:0")

            def run():
                H.D.dsd_stage_verify(ctx, st.w, st.kv, h, None, None, None, B, k, out, lg, 0, 0)

            run()                                             # eager: sizes the workspace
            stream.synchronize()
            out_ref, lg_ref = out.clone(), lg.clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                run()
            stream.synchronize()
            for rep in range(3):
                out.zero_()
                lg.zero_()
                stream.synchronize()
                g.replay()
                stream.synchronize()
                assert torch.equal(out, out_ref) and torch.equal(lg, lg_ref), f"{name}: replay {rep} differs"
                run()                                         # eager work between the replays
                stream.synchronize()


def test_repeated_runs_are_bit_identical_at_128_rows():
    """128 rows take the K-sliced GEMMs with the most slices; the slices are added in a fixed order, so
    the same call on the same inputs gives the same bits every time."""
    B, k = 16, 8
    cfg, m, w, K, V, hid, parent, lens = mini("repeat_m128", B=B, k=k, lens=[40 + 7 * b for b in range(B)], head=True,
                                              V=4112, L=2, d=2048, Hq=16, Hkv=4, F=4096)
    st = H.GpuStage(m, w, B, max(lens) + k + 3)
    st.import_kv(K, V, lens)
    h = st._cast(hid)
    out = torch.empty((B, k, m.d), dtype=torch.bfloat16, device="cuda:0")
    lg = torch.empty((B, k, m.V), dtype=torch.float32, device="cuda:0")
    results = []
    for rep in range(4):
        out.zero_()
        lg.zero_()
        H.D.dsd_stage_verify(st.ctx, st.w, st.kv, h, None, None, None, B, k, out, lg, 0, 0)
        torch.cuda.synchronize()
        results.append((out.clone(), lg.clone()))
    for rep in range(1, 4):
        assert torch.equal(results[rep][0], results[0][0]) and torch.equal(results[rep][1], results[0][1]), f"run {rep} differs"


def test_weights_beyond_the_fp16_range_are_refused():
    """The matrix-core path keeps bf16 projection weights as fp16; a value it cannot hold (beyond 65504,
    infinite, NaN) makes dsd_weights_create fail instead of saturating silently.  Tiny values are fine."""
    cfg, m, w, K, V, hid, parent, lens = mini("range", B=1, k=2, lens=[8])
    w = dict(w)

    def bf16_bits(x):
        return np.uint16(np.float32(x).view(np.uint32) >> 16)

    for bad in (1.0e5, -7.0e4, np.inf, np.nan):
        wb = dict(w)
        wb["l1.wd"] = w["l1.wd"].copy()
        wb["l1.wd"][3, 5] = bf16_bits(bad)
        with pytest.raises(H.D.DsdError, match="65504"):
            H.GpuStage(m, wb, 1, 16)
    ok = dict(w)
    ok["l0.wq"] = w["l0.wq"].copy()
    ok["l0.wq"][0, :4] = [bf16_bits(65280.0), bf16_bits(-65280.0), bf16_bits(2.0 ** -20), bf16_bits(0.0)]
    H.GpuStage(m, ok, 1, 16)


def test_more_than_128_rows_go_through_in_groups_of_sequences():
    """B*k = 168 rows: the library takes the sequences in groups of up to 128 rows (here 16 + 5 sequences
    of 8 rows); the result is checked against the oracle like any other shape."""
    B, k = 21, 8
    check(mini("m168", B=B, k=k, lens=[24 + 5 * (b % 7) for b in range(B)], head=True, V=4112, L=2))


@pytest.mark.parametrize("B,k", [(1, 5), (6, 8)])
def test_outlier_channels_in_the_residual_stream(B, k):
    """Hidden states with a few channels hundreds of times larger than the rest (the massive activations
    of trained decoders): the fp32 residual stream carries them, the fp16 GEMM operands keep their
    relative precision whatever the magnitude, and nothing comes near the fp16 range.  Both GEMM paths
    (5 rows, 48 rows)."""
    cfg, m, w, K, V, hid, parent, lens = mini(f"outliers_{B}x{k}", B=B, k=k, lens=[60 + 11 * b for b in range(B)],
                                              head=True, V=4112, L=2)
    f = O.widen(hid).astype(np.float64)
    f[..., 7] *= 300.0
    f[..., 301] *= -150.0
    f[:, 0, 100] = 800.0
    hid = (f.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)      # truncation to bf16 is good enough for an input
    check((cfg, m, w, K, V, hid, parent, lens))


def test_commit_of_tree_paths_in_the_operand_order_cache():
    """After a tree verify, dsd_kv_commit moves the accepted path's rows (scattered among the k drafted
    slots) to the slots right behind the committed ones.  The bf16 cache keeps K and V in MFMA operand
    order, V with a permutation inside blocks of 32 slots, so the move is checked on exported rows:
    rows exported after the commit equal, bit for bit, the path's rows exported before it; lengths that
    straddle 16- and 32-slot boundaries; one sequence accepts nothing."""
    B, k = 4, 10
    lens = [31, 64, 13, 95]
    cfg, m, w, K, V, hid, parent, _ = mini("commit_tree", B=B, k=k, lens=lens, tree=((3, 2, 2), 10))
    st = H.GpuStage(m, w, B, max(lens) + k + 3)
    st.import_kv(K, V, lens)
    st.verify(hidden=hid, parent=parent)
    par = [int(p) for p in parent]

    def path_to(node):                      # root-to-node path of 1-based node ids
        out = []
        while node:
            out.append(node)
            node = par[node - 1]
        return out[::-1]

    leaves = [n for n in range(1, k + 1) if n not in par]
    paths = [path_to(leaves[0]), path_to(leaves[-1]), [], path_to(par[leaves[-1] - 1])]
    before = [[st.new_rows(l, lens[b], k, B) for b in range(B)] for l in range(m.L)]
    alen = torch.tensor([len(p) for p in paths], dtype=torch.int32, device="cuda:0")
    padded = np.full((B, k), -1, dtype=np.int32)
    for b, p in enumerate(paths):
        padded[b, :len(p)] = p
    H.D.dsd_kv_commit(st.ctx, st.kv, alen, torch.from_numpy(padded).to("cuda:0"), B, k)
    torch.cuda.synchronize()
    assert st.kv.get_len(B) == [lens[b] + len(paths[b]) for b in range(B)]
    for l in range(m.L):
        for b, p in enumerate(paths):
            if not p:
                continue
            gk, gv = st.new_rows(l, lens[b], len(p), B)
            bk, bv = before[l][b]
            idx = [n - 1 for n in p]
            np.testing.assert_array_equal(gk[b], bk[b][:, idx], err_msg=f"K layer {l} sequence {b}")
            np.testing.assert_array_equal(gv[b], bv[b][:, idx], err_msg=f"V layer {l} sequence {b}")
        # committed context untouched
        gk, gv = st.new_rows(l, 0, min(lens), B)
        np.testing.assert_array_equal(gk, O.widen(K[l][:, :, :min(lens)]))
        np.testing.assert_array_equal(gv, O.widen(V[l][:, :, :min(lens)]))

