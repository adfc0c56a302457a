#!/usr/bin/env python3
"""Benchmark of the DSD verify step on one MI355X.

A step is one pass of the whole hot path of a workload: `dsd_stage_verify` over the k drafted rows
of every sequence (plus `dsd_accept` on final-stage workloads), inputs already resident in HBM.

The headline workload (`value`, `roofline`, `cpu_baseline`) is the largest single-GPU
configuration: c4, the Llama-3-70B-shaped stage (10 of 80 layers, batch 8, context 8192, k = 6 chain,
bf16; 19.8 GB of weights and cache per step).  The metric names no configuration of its own, so the
other bf16 configurations are timed in the same run and reported in the same JSON line under
"workloads": c2 (8B middle stage, batch 1), c3 (8B final stage with LM head and adaptive accept,
batch 16), c5 (8B final stage, 32-node draft tree, batch 4).  `--config cN` makes another one the
headline; `--no-others` times the headline alone.  Prints ONE JSON line.
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
TREE_MODES = {"longest": 0, "first": 1, "lossless": 2}


def algorithmic_bytes(cfg):
    """HBM bytes one step has to move: every weight of the block once, every cached K/V element
    once, the appended K/V rows, hidden states in and out, fp32 logits out (final stage); accept:
    one read of the logits rows and of the draft rows."""
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


def golden_lambdas():
    """The frozen thresholds of the key-token rule for the final-stage workloads (the paper calibrates
    them on a validation set and prints no values; these are quantiles of a seeded calibration batch,
    written by tests/golden/calibrate_lambdas.py and used by the parity tests as well)."""
    with open(os.path.join(ROOT, "tests", "golden", "lambdas_8b_final.txt")) as f:
        l1, l2, l3 = [float(x) for x in f.readline().split()]
    return l1, l2, l3


def cpu_baseline(cfg, inp, sample_layers):
    """The oracle, as it stands, on the host cores, on a bounded sample of the same workload: the
    first `sample_layers` layers of the block for all B*k rows, scaled by layers to a full block; on
    final-stage workloads plus the final norm + LM head and the acceptance rule on all rows, timed once
    each at full size."""
    from threadpoolctl import threadpool_info

    from oracle import dsd_oracle as O
    from paper_2511_11733_amd import workloads as W

    L = cfg.model.L
    sample_layers = min(sample_layers or (2 if cfg.model.d > 4096 else L), L)
    weights, K, V, hid, parent = inp["weights"], inp["K"], inp["V"], inp["hid"], inp["parent"]
    m = W.scaled(cfg, L=sample_layers, has_head=False, V=0).model
    reps, dt = 0, 0.0
    while dt < 10.0 and reps < 50:         # about 10-30 s of CPU work
        t0 = time.perf_counter()
        O.stage_forward(m, weights.__getitem__, K[:sample_layers], V[:sample_layers], [cfg.C] * cfg.B, hid, None,
                        parent=parent)
        dt += time.perf_counter() - t0
        reps += 1
    full = dt / reps * L / sample_layers
    sample = (f"{sample_layers} of {L} layers of the same step (all {cfg.B * cfg.k} rows, context {cfg.C}), {reps} "
              f"repetition(s), {dt:.1f} s measured, scaled by layers")
    if cfg.model.has_head:
        mh = W.scaled(cfg, L=0).model          # no layers: final norm + LM head on the rows
        t0 = time.perf_counter()
        O.stage_forward(mh, weights.__getitem__, None, None, [0] * cfg.B, hid, None, parent=parent)
        t_head = time.perf_counter() - t0
        a = inp["accept"]
        t0 = time.perf_counter()
        O.accept(a["logits"].astype(np.float64), a["probs"].astype(np.float64), a["toks"], parent, a["u"],
                 O.AcceptParams(**a["prm"]))
        t_acc = time.perf_counter() - t0
        full += t_head + t_acc
        dt += t_head + t_acc
        sample += f"; plus final norm + LM head ({t_head:.1f} s) and the acceptance rule ({t_acc:.1f} s) on all rows, once each"
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": cfg.B * cfg.k / full, "unit": "tok/s", "cores": int(threads), "kind": "oracle",
            "sample": sample + "; numpy fp64 with multithreaded BLAS matmuls", "seconds_measured": dt}


def dominant_kernel(cfg, kern, per_layer, total_bytes):
    """Name, rocprofv3 name fragment and algorithmic bytes of the launch group the roofline is quoted on:
    the gate/up GEMM (54 % of a layer's weight bytes)."""
    m = cfg.model
    M = cfg.B * cfg.k
    mt = (M + 15) // 16
    mt = {1: 2, 5: 6, 7: 8}.get(mt, mt)
    # computing waves per workgroup as the library picks them: least work on the busiest of the 256 compute units
    twc, best = 4, None
    for t in range(4, 9):
        cost = -(-(-(-(m.F // 16) // t)) // 256) * t
        if best is None or cost <= best:
            twc, best = t, cost
    return ("gateup", per_layer["gateup"],
            f"act_panel_kernel + gemm_tiled_kernel<{mt}, {twc}, TE_SWIGLU> (RMSNorm + gate/up GEMM + SiLU*up; the time "
            "is that of both launches)", f"gemm_tiled_kernel<{mt}, {twc}, 1>")


def committed_traffic(cfg_name, match):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of the same
    bench command (FETCH_SIZE, WRITE_SIZE scaled by the copy-kernel calibration stated in that file).
    Not measured in this run: the counters need a profiler pass of their own."""
    path = os.path.join(ROOT, "profiles", f"verify_step_{cfg_name}.txt")
    if not os.path.exists(path):
        return None, None
    in_counters = False               # the kernel also has a line in the timing table further up
    for line in open(path):
        if line.startswith("HBM byte counters"):
            in_counters = True
        if in_counters and match in line:
            parts = line.split()
            try:
                return (float(parts[-2]) + float(parts[-1])) * 1e6, f"profiles/verify_step_{cfg_name}.txt"
            except ValueError:
                pass
    return None, None


def run_workload(args, name, want_inputs):
    """Times one workload; returns (record, inputs for the CPU leg or None)."""
    import torch

    from paper_2511_11733_amd import dsd as D
    from paper_2511_11733_amd import workloads as W

    cfg = W.CONFIGS[name]
    if args.batch or args.draft_len or args.context:
        # not a benchmark line of its own: the same model and recipe at another row count or context
        assert not (cfg.tree and args.draft_len), "a tree workload keeps its own number of nodes"
        nb, nk, nc = args.batch or cfg.B, args.draft_len or cfg.k, args.context or cfg.C
        cfg = W.scaled(cfg, name=f"{cfg.name} at B={nb} k={nk} C={nc}", B=nb, k=nk, C=nc)
    m = cfg.model
    assert m.dtype == "bf16", "bench workloads are the bf16 configurations"
    dev = "cuda:0"
    B, k, C = cfg.B, cfg.k, cfg.C

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
    tens = [dev_bf16(weights[n]) for n, _, _ in W.weight_specs(m)]
    w = D.Weights(ctx, desc, tens)
    del tens
    torch.cuda.empty_cache()
    kv = D.KVCache(ctx, desc, B, C + k)
    for l in range(m.L):
        kv.import_layer(l, dev_bf16(K[l]), dev_bf16(V[l]))
    kv.set_len([C] * B)
    h_in = dev_bf16(hid)
    h_out = torch.empty_like(h_in)
    mask = depth = par_dev = None
    if parent is not None:
        mask = torch.from_numpy(W.tree_mask_bits(parent).view(np.int64)).to(dev)
        depth = torch.from_numpy(W.tree_depths(parent)).to(dev)
        par_dev = torch.from_numpy(parent).to(dev)
    logits = probs = toks = unif = alen = nxt = path = prm = None
    prm_kw = None
    if m.has_head:
        # [B, k+1, V]: row 0 is the root row (one untimed 1-row pass on the pending row, then committed),
        # rows 1..k are written by the timed k-row pass
        logits = torch.zeros((B, k + 1, m.V), dtype=torch.float32, device=dev)
        alen = torch.zeros(B, dtype=torch.int32, device=dev)
        nxt = torch.zeros(B, dtype=torch.int32, device=dev)
        path = torch.zeros((B, k), dtype=torch.int32, device=dev)
        l1, l2, l3 = golden_lambdas()
        prm_kw = dict(lambda1=l1, lambda2=l2, lambda3=l3, tau=cfg.tau, top_m=cfg.top_m, temperature=args.temperature,
                      tree_mode=TREE_MODES[args.tree_mode])
        prm = D.accept_params(**prm_kw)

    def stage():
        D.dsd_stage_verify(ctx, w, kv, h_in, None, mask, depth, B, k, h_out, logits,
                           (k + 1) * m.V if m.has_head else 0, m.V if m.has_head else 0)

    def step():
        stage()
        if m.has_head:
            D.dsd_accept(ctx, logits, probs, toks, par_dev, unif, prm, B, k, m.V, alen, nxt, path)

    with torch.cuda.stream(stream):
        if m.has_head:
            # the root row: the pending token's row at position C-1, verified alone and committed
            root_h = dev_bf16(W.make_hidden(cfg, rows=1, tag="root"))
            kv.set_len([C - 1] * B)
            D.dsd_stage_verify(ctx, w, kv, root_h, None, None, None, B, 1, None, logits, (k + 1) * m.V, 0)
            D.dsd_kv_commit(ctx, kv, torch.ones(B, dtype=torch.int32, device=dev), None, B, 1)
            stage()
            stream.synchronize()
            assert kv.get_len(B) == [C] * B
            # the synthetic draft of the workload recipe: q_p = softmax(target row p + N(0, 0.5^2)), children
            # of p drawn from q_p without replacement
            noise = torch.from_numpy(W.make_draft_noise(cfg, k + 1, m.V)).to(dev)
            probs = torch.softmax(logits + noise, dim=-1).contiguous()
            del noise
            par_list = list(range(k)) if parent is None else [int(p) for p in parent]
            gen = torch.Generator(device=dev)
            gen.manual_seed(cfg.seed)
            toks = torch.zeros((B, k), dtype=torch.int64, device=dev)
            rows = torch.arange(B, device=dev)
            for i in range(k):
                pr = probs[:, par_list[i]].clone()
                for j in range(i):
                    if par_list[j] == par_list[i]:
                        pr[rows, toks[:, j]] = 0.0
                toks[:, i] = torch.multinomial(pr, 1, generator=gen)[:, 0]
            toks = toks.to(torch.int32).contiguous()
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

        probe = None
        if want_inputs and not args.no_stream_probe:
            # what a bare stream reaches on this chip, for context: one kernel that only reads 1 GiB, one that copies it
            buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
            buf.zero_()
            stream.synchronize()
            probe = {"bytes": 1 << 30, "read_GBps": (1 << 30) / ctx.stream_probe(buf, 0, 10) / 1e6,
                     "read_nontemporal_GBps": (1 << 30) / ctx.stream_probe(buf, 3, 10) / 1e6,
                     "read_one_stream_per_wave_GBps": (1 << 30) / ctx.stream_probe(buf, 2, 10) / 1e6,
                     "copy_read_plus_write_GBps": (1 << 30) / ctx.stream_probe(buf, 1, 10) / 1e6,
                     "measured": "hip events on the library stream, average of 10 launches after 2 warm-up launches"}
            del buf

    if args.copy_calibration:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    total_bytes, per_layer, head_bytes, accept_bytes = algorithmic_bytes(cfg)
    kern = {kc: (t / n if n else 0.0) for kc, (t, n) in prof.items()}
    dominant, dom_bytes, dom_name, dom_match = dominant_kernel(cfg, kern, per_layer, total_bytes)
    dom_ms = kern[dominant]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    traffic, traffic_src = committed_traffic(cfg.name, dom_match)
    step_gbps = (total_bytes + accept_bytes) / (ms * 1e-3) / 1e9
    rec = {
        "workload": f"{cfg.name}: {m.name} L={m.L} d={m.d} heads={m.Hq}/{m.Hkv} F={m.F} V={m.V} "
                    f"B={B} C={C} k={k} {'tree' if cfg.tree else 'chain'}"
                    + (f" accept={args.tree_mode}" if m.has_head and args.tree_mode != "longest" else "")
                    + (f" T={args.temperature:g}" if m.has_head and args.temperature != 1.0 else ""),
        "ms_per_step": ms,
        "verified_tokens_per_s": B * k / (ms * 1e-3),
        "step_latency_ms_p10_p50_p90": [round(pct[10], 5), round(pct[50], 5), round(pct[90], 5)],
        "committed_tokens_per_s": committed,
        "stage_algorithmic_GB": total_bytes / 1e9,
        "accept_algorithmic_GB": accept_bytes / 1e9,
        "stage_achieved_GBps": step_gbps,
        "stage_frac_of_hbm_peak": step_gbps / HBM_PEAK_GBPS,
        "kernel_avg_ms": {kc: round(v, 5) for kc, v in kern.items() if v},
        "kernel_launches_per_step": {kc: n // args.steps for kc, (t, n) in prof.items() if n},
        "head_us": round(kern.get("head", 0.0) * 1e3, 2) if m.has_head else None,
        "accept_us": round(kern.get("accept", 0.0) * 1e3, 2) if m.has_head else None,
        "input_generation_s": round(t_gen, 1),
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_src,
                     "bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms,
                     "step_frac": step_gbps / HBM_PEAK_GBPS,
                     "measured": "hip events on the library stream, second pass of the same steps"},
    }
    if probe:
        rec["stream_probe"] = probe
    inputs = None
    if want_inputs:
        inputs = dict(weights=weights, K=K, V=V, hid=hid, parent=parent)
        if m.has_head:
            inputs["accept"] = dict(logits=logits.cpu().numpy(), probs=probs.cpu().numpy(), toks=toks.cpu().numpy(),
                                    u=unif.cpu().numpy(),
                                    prm={kk: vv for kk, vv in prm_kw.items()})
    # give the device memory back before the next workload
    del logits, probs, h_in, h_out
    kv.close()
    w.close()
    ctx.close()
    torch.cuda.empty_cache()
    return cfg, rec, inputs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c4", help="headline workload: c4 (default), c2, c3, c5")
    ap.add_argument("--no-others", action="store_true", help="time the headline workload only")
    ap.add_argument("--tree-mode", default="longest", choices=sorted(TREE_MODES),
                    help="dsd_accept's tree rule (final-stage workloads); lossless = recursive rejection over siblings")
    ap.add_argument("--temperature", type=float, default=1.0, help="dsd_accept's temperature; 0 = greedy verification")
    ap.add_argument("--batch", type=int, default=0, help="row-count sweeps: the named workload with another batch size")
    ap.add_argument("--draft-len", type=int, default=0, help="row-count sweeps: another number of drafted rows (chains only)")
    ap.add_argument("--context", type=int, default=0, help="context sweeps: another committed length per sequence")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stream-probe", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (a known-size reference for HBM byte counters)")
    ap.add_argument("--cpu-sample-layers", type=int, default=0, help="0 = all layers at d_model 4096, 2 beyond")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the verify step of ONE node); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    sweep = bool(args.batch or args.draft_len or args.context)
    cfg, head, inputs = run_workload(args, args.config, want_inputs=True)
    out = {
        "metric": "verified_tokens_per_s", "value": head["verified_tokens_per_s"], "unit": "tok/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": head["workload"]},
        "verify_step_latency_ms": head["ms_per_step"],
    }
    for key in ("step_latency_ms_p10_p50_p90", "committed_tokens_per_s", "stage_algorithmic_GB", "stage_achieved_GBps",
                "stage_frac_of_hbm_peak", "kernel_avg_ms", "kernel_launches_per_step", "head_us", "accept_us",
                "input_generation_s", "stream_probe", "roofline"):
        if key in head:
            out[key] = head[key]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inputs, args.cpu_sample_layers)
    del inputs
    if not args.no_others and not sweep:
        # the other bf16 configurations, same run, same protocol (no CPU leg: that belongs to the headline)
        others = {}
        for name in ("c2", "c3", "c4", "c5"):
            if name == args.config:
                continue
            _, rec, _ = run_workload(args, name, want_inputs=False)
            others[name] = {kk: rec[kk] for kk in ("workload", "ms_per_step", "verified_tokens_per_s", "committed_tokens_per_s",
                                                  "stage_algorithmic_GB", "stage_frac_of_hbm_peak", "kernel_avg_ms",
                                                  "head_us", "accept_us")}
            others[name]["dominant_kernel_frac_of_hbm_peak"] = rec["roofline"]["frac"]
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
