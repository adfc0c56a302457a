#!/usr/bin/env python3
"""Benchmark of the DSD verify step on one MI355X.

A step is one pass of the whole hot path of the named workload: `dsd_stage_verify` over the
k drafted rows of every sequence (plus `dsd_accept` on final-stage workloads), inputs already
resident in HBM.  The default workload is the Llama-3-8B-shaped middle stage (8 of 32 layers,
batch 1, context 2048, k = 5 chain draft, bf16), the configuration the headline metric is
quoted on.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def algorithmic_bytes(cfg):
    """HBM bytes one step has to move: every weight of the block once, every cached K/V element
    once, the appended K/V rows, hidden states in and out, fp32 logits out (final stage)."""
    m = cfg.model
    es = 2 if m.dtype == "bf16" else 4
    qd, kd = m.Hq * m.hd, m.Hkv * m.hd
    per_layer = {
        "qkv": (qd + 2 * kd) * m.d * es + m.d * es,
        "oproj": m.d * qd * es,
        "gateup": 2 * m.F * m.d * es + m.d * es,
        "down": m.d * m.F * es,
        "attn": 2 * cfg.B * kd * cfg.C * es,
    }
    M = cfg.B * cfg.k
    total = m.L * sum(per_layer.values())
    total += m.L * 2 * M * kd * es            # appended K/V rows
    total += 2 * M * m.d * es                 # hidden in + out
    head = 0
    if m.has_head:
        head = m.V * m.d * es + m.d * es + M * m.V * 4
        total += head
    accept = 2 * cfg.B * (cfg.k + 1) * m.V * 4 if m.has_head else 0
    return total, per_layer, head, accept


def cpu_baseline(cfg, weights, K, V, hid, parent, sample_layers):
    """The oracle, as it stands, on the host cores, on a bounded sample of the same workload: the
    first `sample_layers` layers of the block for all B*k rows; scaled to tokens/s of a full step."""
    from threadpoolctl import threadpool_info

    from oracle import dsd_oracle as O
    from paper_2511_11733_amd import workloads as W

    sample_layers = sample_layers or cfg.model.L
    m = W.scaled(cfg, L=sample_layers, has_head=False, V=0).model
    reps, dt = 0, 0.0
    while dt < 10.0 and reps < 50:         # about 10-30 s of CPU work
        t0 = time.perf_counter()
        O.stage_forward(m, weights.__getitem__, K[:sample_layers], V[:sample_layers], [cfg.C] * cfg.B, hid, None,
                        parent=parent)
        dt += time.perf_counter() - t0
        reps += 1
    full = dt / reps * cfg.model.L / sample_layers
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": cfg.B * cfg.k / full, "unit": "tok/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{sample_layers} of {cfg.model.L} layers of the same step (all {cfg.B * cfg.k} rows, context "
                      f"{cfg.C}), {reps} repetition(s), {dt:.1f} s measured, scaled by layers; numpy fp64 with multithreaded BLAS matmuls",
            "seconds_measured": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2", help="workload: c2 (default), c3, c4, c5")
    ap.add_argument("--tree-mode", default="longest", choices=["longest", "first", "lossless"],
                    help="dsd_accept's tree rule (final-stage workloads); lossless = recursive rejection over siblings")
    ap.add_argument("--temperature", type=float, default=1.0, help="dsd_accept's temperature; 0 = greedy verification")
    ap.add_argument("--batch", type=int, default=0, help="row-count sweeps: the named workload with another batch size")
    ap.add_argument("--draft-len", type=int, default=0, help="row-count sweeps: another number of drafted rows (chains only)")
    ap.add_argument("--context", type=int, default=0, help="context sweeps: another committed length per sequence")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (a known-size reference for HBM byte counters)")
    ap.add_argument("--cpu-sample-layers", type=int, default=0, help="0 = all layers of the block")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the verify step of ONE node); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2511_11733_amd import dsd as D
    from paper_2511_11733_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config]
    if args.batch or args.draft_len or args.context:
        # not a benchmark line of its own: the same model and recipe at another row count or context
        assert not (cfg.tree and args.draft_len), "a tree workload keeps its own number of nodes"
        nb, nk, nc = args.batch or cfg.B, args.draft_len or cfg.k, args.context or cfg.C
        cfg = W.scaled(cfg, name=f"{cfg.name} at B={nb} k={nk} C={nc}", B=nb, k=nk, C=nc)
    m = cfg.model
    assert m.dtype == "bf16", "bench workloads are the bf16 configurations"
    dev = "cuda:0"

    t_gen = time.perf_counter()
    weights = W.make_weights(m, cfg.seed, threads=16)
    K, V = W.make_kv(cfg, threads=16)
    hid = W.make_hidden(cfg)
    parent = W.ranked_tree_parents() if cfg.tree else None
    t_gen = time.perf_counter() - t_gen

    def dev_bf16(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    stream = torch.cuda.Stream()
    ctx = D.Context(0, stream)
    desc = D.model_desc(m)
    tens = [dev_bf16(weights[name]) for name, _, _ in W.weight_specs(m)]
    w = D.Weights(ctx, desc, tens)
    del tens
    torch.cuda.empty_cache()
    kv = D.KVCache(ctx, desc, cfg.B, cfg.C + cfg.k)
    for l in range(m.L):
        kv.import_layer(l, dev_bf16(K[l]), dev_bf16(V[l]))
    kv.set_len([cfg.C] * cfg.B)
    h_in = dev_bf16(hid)
    h_out = torch.empty_like(h_in)
    B, k = cfg.B, cfg.k
    mask = depth = par_dev = None
    if parent is not None:
        mask = torch.from_numpy(W.tree_mask_bits(parent).view(np.int64)).to(dev)
        depth = torch.from_numpy(W.tree_depths(parent)).to(dev)
        par_dev = torch.from_numpy(parent).to(dev)
    logits = probs = toks = unif = alen = nxt = path = prm = None
    if m.has_head:
        # [B, k+1, V]: row 0 is the root row (produced once, untimed, by a 1-row pass on a pending
        # row), rows 1..k are written by the timed k-row pass
        logits = torch.zeros((B, k + 1, m.V), dtype=torch.float32, device=dev)
        alen = torch.zeros(B, dtype=torch.int32, device=dev)
        nxt = torch.zeros(B, dtype=torch.int32, device=dev)
        path = torch.zeros((B, k), dtype=torch.int32, device=dev)
        prm = D.accept_params(lambda1=1.05, lambda2=2e-5, lambda3=0.3, tau=cfg.tau, top_m=cfg.top_m, temperature=args.temperature,
                              tree_mode={"longest": 0, "first": 1, "lossless": 2}[args.tree_mode])

    def stage():
        D.dsd_stage_verify(ctx, w, kv, h_in, None, mask, depth, B, k, h_out, logits,
                           (k + 1) * m.V if m.has_head else 0, m.V if m.has_head else 0)

    def step():
        stage()
        if m.has_head:
            D.dsd_accept(ctx, logits, probs, toks, par_dev, unif, prm, B, k, m.V, alen, nxt, path)

    with torch.cuda.stream(stream):
        if m.has_head:
            stage()
            stream.synchronize()
            logits[:, 0] = logits[:, 1]          # stand-in root row (timing only)
            noise = torch.from_numpy(W.make_draft_noise(cfg, k + 1, m.V)).to(dev)
            probs = torch.softmax(logits + noise, dim=-1).contiguous()
            del noise
            par_list = list(range(k)) if parent is None else [int(p) for p in parent]
            toks = torch.stack([torch.multinomial(probs[:, par_list[i]], 1)[:, 0] for i in range(k)], dim=1).to(torch.int32).contiguous()
            unif = torch.from_numpy(W.make_uniforms(cfg, k + 1)).to(dev)
        for _ in range(args.warmup):
            step()
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = (t1 - t0) * 1e3 / args.steps

        # spread of the step latency: event pairs around every step of one more pass (the events sit on
        # the library's stream, which is torch's current stream here)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for e0, e1 in evs:
            e0.record()
            step()
            e1.record()
        stream.synchronize()
        lat = np.sort(np.array([e0.elapsed_time(e1) for e0, e1 in evs]))
        pct = {q: float(lat[min(len(lat) - 1, int(round(q / 100.0 * (len(lat) - 1))))]) for q in (10, 50, 90)}
        committed = None
        if m.has_head:
            committed = float((alen.sum().item() + B)) / (ms * 1e-3)    # accepted tokens + the extra one per sequence

        # per-kernel-class durations from HIP events on the library's stream: a second pass over the
        # same K steps (the events cost a little per launch, so the timed region above runs without)
        ctx.profile_enable(True)
        for _ in range(args.steps):
            step()
        prof = ctx.profile_read()
        ctx.profile_enable(False)

    if args.copy_calibration:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    total_bytes, per_layer, head_bytes, accept_bytes = algorithmic_bytes(cfg)
    kern = {kc: (t / n if n else 0.0) for kc, (t, n) in prof.items()}
    if kern.get("stage", 0.0) > 0.0:
        # the opt-in persistent form (at most 8 rows): the whole block of layers is one kernel
        dominant, dom_bytes = "stage", total_bytes
        dom_name = "stage_persist_kernel (all layers of the block: QKV, attention, O-proj, gate/up, down)"
        dom_match = "stage_persist_kernel"
    else:
        dominant, dom_bytes = "gateup", per_layer["gateup"]
        M = B * k
        if M <= 10:      # the library's switch-over between its two GEMM paths
            dom_name = "gemm_skinny_kernel<1, 2, A_F32_GAIN, EPI_SWIGLU, 4> (RMSNorm + gate/up GEMM + SiLU*up, one launch)"
            dom_match = "gemm_skinny_kernel<1, 2, 0, 1"
        else:
            # the step is the activation pre-pass (a few us) plus the weight-streaming GEMM; the
            # library picks the GEMM's geometry from the row count and the matrix width
            mt = (M + 15) // 16
            mt = {1: 2, 5: 6, 7: 8}.get(mt, mt)
            twc = 8 if -(-(2 * (m.F // 16)) // 16) * 5 >= 256 * 4 else 4
            dom_name = (f"act_panel_kernel + gemm_tiled_kernel<{mt}, {twc}, TE_SWIGLU> (RMSNorm + gate/up GEMM + SiLU*up; "
                        "the time is that of both launches)")
            dom_match = f"gemm_tiled_kernel<{mt}, {twc}, 1>"
    dom_ms = kern[dominant]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    traffic = None
    prof_txt = os.path.join(ROOT, "profiles", f"verify_step_{cfg.name}.txt")
    if os.path.exists(prof_txt):
        # HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
        # (FETCH_SIZE, WRITE_SIZE scaled by the copy-kernel calibration stated in that file)
        for line in open(prof_txt):
            if dom_match in line:
                parts = line.split()
                try:
                    traffic = (float(parts[-2]) + float(parts[-1])) * 1e6
                except ValueError:
                    pass
    roofline = {"bound": "hbm", "kernel": dom_name,
                "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                "traffic": traffic, "bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms,
                "measured": "hip events on the library stream, second pass of the same steps"}
    out = {
        "metric": "verified_tokens_per_s", "value": B * k / (ms * 1e-3), "unit": "tok/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {m.name} L={m.L} d={m.d} heads={m.Hq}/{m.Hkv} F={m.F} V={m.V} "
                               f"B={B} C={cfg.C} k={k} {'tree' if cfg.tree else 'chain'}"
                               + (f" accept={args.tree_mode}" if m.has_head and args.tree_mode != "longest" else "")
                               + (f" T={args.temperature:g}" if m.has_head and args.temperature != 1.0 else "")},
        "verify_step_latency_ms": ms,
        "step_latency_ms_p10_p50_p90": [round(pct[10], 5), round(pct[50], 5), round(pct[90], 5)],
        "committed_tokens_per_s": committed,
        "stage_algorithmic_GB": total_bytes / 1e9,
        "stage_achieved_GBps": (total_bytes + accept_bytes) / (ms * 1e-3) / 1e9,
        "stage_frac_of_hbm_peak": (total_bytes + accept_bytes) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "kernel_avg_ms": {kc: round(v, 5) for kc, v in kern.items() if v},
        "kernel_launches_per_step": {kc: n // args.steps for kc, (t, n) in prof.items() if n},
        "input_generation_s": round(t_gen, 1),
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, weights, K, V, hid, parent, args.cpu_sample_layers)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
