#!/usr/bin/env python3
"""Benchmark of the EasySpec draft hot path on one MI355X.

One "step" is one drafting iteration of the three-stage loop: bonus calibration over gamma+1
tokens (which also yields the first draft token), gamma-1 layer-parallel fuzzy draft steps,
and greedy acceptance against a synthetic verifier output.  `value` is drafted tokens per
second over whole iterations (gamma tokens per iteration); the per-call figures the metric
names (fuzzy draft-step tokens/s, calibration microseconds, each with its share of the HBM
roofline) are reported in the same JSON line.

Inputs are seeded and synthetic: random-init weights of the named shape, a synthetic KV prefix
standing in for a prefilled context, uniform random token ids.  Everything is resident in HBM
before the timed region starts.
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

HBM_PEAK_GBS = 8000.0
# HBM KiB per launch of the dominant kernel (gate/up projection) from the rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs summarised in profiles/hbm_traffic_llama3_8b_ctx2048.md (scaled by a 1 GiB copy).
MEASURED_TRAFFIC_KIB = {"llama3_8b_ctx2048": 230288.8}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def batched_step(args, wl, torch, synth, es):
    """The batched long-context workload (a parity case, not the headline): times the fuzzy draft step alone,
    all sequences in one launch sequence.  The KV prefix is drawn on the device (its values do not matter for
    the time); parity of this case is covered by tests/test_gpu_shapes.py at reduced depth."""
    cfg = synth.model_shape(wl["model"], **({"n_layers": args.layers} if args.layers else {}))
    ctxs = [int(c) for c in wl["context"]]
    B = len(ctxs)
    L, hkv, hd = cfg["n_layers"], cfg["n_kv_heads"], cfg["head_dim"]
    policy = es.EASYSPEC_POLICY_ALIGNED if wl["group_policy"] == "aligned" else es.EASYSPEC_POLICY_PACKED
    bounds = es.easyspec_default_groups(L, args.group_size or wl["group_size"], policy)
    weights = synth.make_weights(cfg, args.seed)
    dev = torch.device("cuda:0")
    ctx = es.easyspec_create(es.make_config(cfg, B, max(ctxs) + 64, 16), torch.cuda.current_stream().cuda_stream)
    es.easyspec_load_weights(ctx, weights)
    es.easyspec_set_groups(ctx, bounds)
    gen = torch.Generator(device=dev).manual_seed(args.seed)
    for b, n in enumerate(ctxs):
        k = torch.randn(L, hkv, n, hd, device=dev, generator=gen).to(torch.bfloat16).view(torch.int16)
        v = torch.randn(L, hkv, n, hd, device=dev, generator=gen).to(torch.bfloat16).view(torch.int16)
        es.easyspec_kv_import(ctx, b, k, v, n)
        del k, v
    tok = torch.zeros(B, dtype=torch.int32, device=dev)

    def steps(n):
        for i in range(n):
            if i % (wl["gamma"] - 1) == 0:          # a drafting iteration's fuzzy slots, then back to the prefix
                for b, c in enumerate(ctxs):
                    es.easyspec_truncate(ctx, b, c)
            es.easyspec_draft_step(ctx, tok, tok, None)

    steps(args.warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    steps(args.steps)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    for b, c in enumerate(ctxs):
        es.easyspec_truncate(ctx, b, c)
    step_bytes = int(es.easyspec_step_bytes(ctx))
    es.easyspec_destroy(ctx)
    achieved = step_bytes / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "draft tokens/sec (batched fuzzy draft step, all sequences)", "value": round(B / (ms * 1e-3), 2),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (weights from the seeded generator, KV prefix drawn on the device)",
        "config": {"workload": args.workload, "shape": wl["model"], "contexts": ctxs, "batch": B,
                   "group_size": args.group_size or wl["group_size"], "sets": [int(x) for x in bounds]},
        "draft_step": {"us": round(ms * 1e3, 1), "bytes": step_bytes, "hbm_frac": round(achieved / HBM_PEAK_GBS, 4)},
        "roofline": {"bound": "hbm", "kernel": "whole draft step", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None},
        "cpu_baseline": None}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama3_8b_ctx2048")
    ap.add_argument("--seed", type=int, default=2025)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging; makes the result invalid)")
    ap.add_argument("--group-size", type=int, default=0, help="override the workload's layer-parallel size N (1 = sequential)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the oracle baseline leg")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (a kernel of known traffic, to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--traffic-kib", type=float, default=None,
                    help="HBM KiB per launch of the dominant kernel from rocprofv3 --pmc runs (default: the committed figure)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import easyspec_synth as synth
    import paper_2502_02493_amd as es

    if not torch.cuda.is_available():
        print("bench.py: no HIP device visible", file=sys.stderr)
        sys.exit(3)
    es.load_library()
    wl = dict(synth.WORKLOADS[args.workload])
    if isinstance(wl["context"], tuple):
        batched_step(args, wl, torch, synth, es)
        return
    over = {"n_layers": args.layers} if args.layers else {}
    if args.group_size:
        wl["group_size"] = args.group_size
    cfg = synth.model_shape(wl["model"], **over)
    gamma, ctx_len, B = wl["gamma"], wl["context"], 1
    M = gamma + 1
    policy = es.EASYSPEC_POLICY_ALIGNED if wl["group_policy"] == "aligned" else es.EASYSPEC_POLICY_PACKED
    bounds = es.easyspec_default_groups(cfg["n_layers"], wl["group_size"], policy)
    max_ctx = ctx_len + M + max(gamma, 4 * 12) + 8      # room for the chain and for the widest tree timed below

    t0 = time.time()
    weights = synth.make_weights(cfg, args.seed)
    kpre, vpre = synth.make_kv_prefix(cfg, args.seed + 1, ctx_len)
    log(f"[bench] synthetic inputs drawn in {time.time() - t0:.1f}s")

    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    ctx = es.easyspec_create(es.make_config(cfg, B, max_ctx, 16), stream)
    t0 = time.time()
    es.easyspec_load_weights(ctx, weights)
    es.easyspec_set_groups(ctx, bounds)
    es.easyspec_kv_import(ctx, 0, kpre, vpre, ctx_len)
    log(f"[bench] weights packed and KV prefix imported in {time.time() - t0:.1f}s")

    calib_tok = torch.from_numpy(synth.make_tokens(args.seed + 2, 16, cfg["vocab"]).reshape(1, 16)).to(dev)
    n_tok = np.array([M], np.int32)
    draft = torch.zeros(gamma + 1, dtype=torch.int32, device=dev)      # draft[j] = j-th drafted token
    target = torch.from_numpy(synth.make_tokens(args.seed + 3, gamma + 1, cfg["vocab"]).reshape(1, gamma + 1)).to(dev)
    acc = torch.zeros(1, dtype=torch.int32, device=dev)
    bonus = torch.zeros(1, dtype=torch.int32, device=dev)
    esz = 4
    dptr = draft.data_ptr()

    # Calibration length per iteration: gamma + 1 tokens (every drafted token accepted, the costliest case), or,
    # for the calibration-dominant workload, accepted-length + 1 with the accepted length drawn uniformly from
    # 0 .. gamma by the seeded generator (partial rewrites of the fuzzy slots).
    draw_m = wl.get("calib_tokens") == "uniform"
    m_rng = np.random.Generator(np.random.Philox(key=[args.seed, 77]))
    m_used = []
    n_tok_iter = n_tok.copy()

    def iteration(ev=None):
        es.easyspec_truncate(ctx, 0, ctx_len)
        if draw_m:
            n_tok_iter[0] = int(m_rng.integers(1, M + 1))
        if ev:
            m_used.append(int(n_tok_iter[0]))
            ev[0].record()
        es.easyspec_calibrate(ctx, calib_tok, n_tok_iter, dptr, None, 0)  # first draft token -> draft[0]
        if ev: ev[1].record()
        for j in range(1, gamma):
            es.easyspec_draft_step(ctx, dptr + (j - 1) * esz, dptr + j * esz, None)
        if ev: ev[2].record()
        es.easyspec_greedy_accept(dptr, target, 1, gamma, acc, bonus, stream)

    if args.copy_mib:
        src = torch.ones(args.copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads and writes copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        iteration()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        iteration(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    calib_us = 1e3 * float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    step_us = 1e3 * float(np.mean([e[1].elapsed_time(e[2]) for e in evs])) / (gamma - 1)

    # algorithmic bytes (weights once + the KV slots read)
    es.easyspec_truncate(ctx, 0, ctx_len)
    step_bytes = es.easyspec_step_bytes(ctx)              # one draft step at this context
    e = 2 if cfg["dtype"] == "bf16" else 4
    m_mean = float(np.mean(m_used)) if m_used else float(M)
    calib_bytes = step_bytes + (m_mean - 1) * cfg["n_layers"] * 2 * cfg["n_kv_heads"] * cfg["head_dim"] * e
    gu_bytes = 2 * cfg["d_ffn"] * cfg["d_model"] * e

    # dominant kernel (gate/up projection: 2*F*d weights per launch), HIP events around each launch,
    # same iteration sequence again
    n_launch = args.steps * gamma * cfg["n_layers"]
    es.easyspec_profile_begin(ctx, es.EASYSPEC_OP_GATEUP, n_launch)
    for k in range(args.steps):
        iteration()
    n_timed, total_ms = es.easyspec_profile_end(ctx)
    # an event pair with nothing between still spans the gap between two stream markers: measure that
    # gap the same way and take it off, so that the figure is the kernel's own duration
    null = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
    es.easyspec_draft_step(ctx, dptr, dptr + esz, None)
    for a_, b_ in null:
        a_.record(); b_.record()
    torch.cuda.synchronize()
    null_ms = float(np.median([a_.elapsed_time(b_) for a_, b_ in null]))
    gu_raw_ms = total_ms / max(n_timed, 1)
    gu_ms = gu_raw_ms - null_ms
    gu_gbs = gu_bytes / (gu_ms * 1e-3) / 1e9
    per_op = {}
    for name, op in (("qkv", es.EASYSPEC_OP_QKV), ("attn", es.EASYSPEC_OP_ATTN), ("oproj", es.EASYSPEC_OP_OPROJ),
                     ("down", es.EASYSPEC_OP_DOWN), ("head", es.EASYSPEC_OP_HEAD)):
        es.easyspec_profile_begin(ctx, op, 4096)
        iteration()
        n_, ms_ = es.easyspec_profile_end(ctx)
        per_op[name + "_us_per_iteration"] = round(1e3 * ms_, 1)
    per_op["gateup_us_per_iteration"] = round(1e3 * gu_ms * gamma * cfg["n_layers"], 1)

    # acceptance by speculative sampling (temperature 0.8, the paper's second setting) on logits of
    # this vocabulary: reported beside the greedy iteration, not part of `value`
    V = cfg["vocab"]
    tl = torch.from_numpy(synth.make_logits(args.seed + 5, gamma + 1, V)).to(dev)
    dl = (tl[:gamma] + 0.7 * torch.from_numpy(synth.make_logits(args.seed + 6, gamma, V, std=1.0)).to(dev)).contiguous()
    ru = torch.from_numpy(synth.make_uniforms(args.seed + 7, gamma + 1)).to(dev)
    ws = torch.empty(es.easyspec_accept_workspace_bytes(1, gamma, V) // 8, dtype=torch.float64, device=dev)
    sa = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    n_acc = 50
    for k in range(n_acc + 5):
        if k == 5: sa[0].record()
        es.easyspec_accept(draft, dl, tl, ru, ru[gamma:], 1, gamma, V, 0.8, acc, bonus, ws, stream)
    sa[1].record()
    torch.cuda.synchronize()
    accept_us = 1e3 * sa[0].elapsed_time(sa[1]) / n_acc

    # one level of a token tree per forward (tree widths of the paper's ablation), same context
    tree = {}
    W = es.EASYSPEC_MAX_TREE_WIDTH
    tree_in = torch.from_numpy(synth.make_tokens(args.seed + 8, W, cfg["vocab"]).reshape(1, W)).to(dev)
    tree_out = torch.zeros(1, W, dtype=torch.int32, device=dev)
    for width in (4, 8, 12):
        levels = 4
        evs_t = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        reps = max(2, args.steps // 4)
        tot = 0.0
        for rep in range(reps + 1):
            es.easyspec_truncate(ctx, 0, ctx_len)
            es.easyspec_calibrate(ctx, calib_tok, n_tok, dptr, None, 0)
            evs_t[0].record()
            for lvl in range(levels):
                par = np.full((1, W), -1, np.int32)
                if lvl:
                    par[0, :width] = (lvl - 1) * width + np.arange(width) // 2      # two children per node, half the nodes are leaves
                es.easyspec_draft_tree_step(ctx, tree_in, np.array([width], np.int32), par, tree_out, None)
            evs_t[1].record()
            torch.cuda.synchronize()
            if rep:
                tot += evs_t[0].elapsed_time(evs_t[1])
        us = 1e3 * tot / (reps * levels)
        tree[f"width_{width}"] = {"us_per_level": round(us, 1), "hbm_frac": round(step_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    es.easyspec_truncate(ctx, 0, ctx_len)

    # the full-layer-parallel ablation (paper App. B) on the same sets: 6 launches per set instead of 4 + 2k
    es.easyspec_set_parallel_mode(ctx, es.EASYSPEC_PARALLEL_FULL_LAYER)
    fl = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    reps = max(2, args.steps // 4)
    tot = 0.0
    for rep in range(reps + 1):
        es.easyspec_truncate(ctx, 0, ctx_len)
        es.easyspec_calibrate(ctx, calib_tok, n_tok, dptr, None, 0)
        fl[0].record()
        for j in range(1, gamma):
            es.easyspec_draft_step(ctx, dptr + (j - 1) * esz, dptr + j * esz, None)
        fl[1].record()
        torch.cuda.synchronize()
        if rep:
            tot += fl[0].elapsed_time(fl[1])
    full_us = 1e3 * tot / (reps * (gamma - 1))
    es.easyspec_set_parallel_mode(ctx, es.EASYSPEC_PARALLEL_ATTENTION)
    es.easyspec_truncate(ctx, 0, ctx_len)

    # what a kernel that only reads reaches on this device (same loads as the weight stream), 4 GiB per pass
    probe = torch.empty(1 << 30, dtype=torch.int32, device=dev)
    probe.zero_()
    sink = torch.empty(es.easyspec_stream_read_sink_floats(), dtype=torch.float32, device=dev)
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for k in range(8):
        if k == 3: pe[0].record()
        es.easyspec_stream_read(probe, probe.numel() * 4, sink, stream)
    pe[1].record()
    torch.cuda.synchronize()
    stream_gbs = 5 * probe.numel() * 4 / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e9
    del probe

    traffic_kib = args.traffic_kib if args.traffic_kib is not None else (
        None if args.layers else MEASURED_TRAFFIC_KIB.get(args.workload))
    out = {
        "metric": "draft tokens/sec (whole drafting iteration: calibration + fuzzy steps + accept)",
        "value": round(gamma * args.steps / wall, 2),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * wall / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload + ("" if not args.layers else f"_L{args.layers}_INVALID"),
                   "shape": cfg["name"], "context": ctx_len, "batch": B,
                   "group_size": wl["group_size"], "sets": [int(x) for x in bounds], "gamma": gamma, "calib_tokens": M},
        "draft_step": {"us": round(step_us, 1), "tokens_per_s": round(1e6 / step_us, 2), "bytes": int(step_bytes),
                       "hbm_frac": round(step_bytes / (step_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                       "frac_of_stream_read": round(step_bytes / (step_us * 1e-6) / 1e9 / stream_gbs, 4)},
        "calibrate": {"us": round(calib_us, 1), "tokens": M if not draw_m else round(m_mean, 2),
                      "tokens_drawn": "uniform 1..%d" % M if draw_m else "fixed", "bytes": int(calib_bytes),
                      "hbm_frac": round(calib_bytes / (calib_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
        "roofline": {"bound": "hbm", "kernel": "gateup_kernel", "achieved": round(gu_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gu_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic_kib * 1024 if traffic_kib else None,
                     "bytes_per_launch": int(gu_bytes), "avg_launch_us": round(1e3 * gu_ms, 2),
                     "event_pair_us": round(1e3 * gu_raw_ms, 2), "empty_event_pair_us": round(1e3 * null_ms, 2),
                     "launches_timed": n_timed, "stream_read_gbs": round(stream_gbs, 1),
                     "frac_of_stream_read": round(gu_gbs / stream_gbs, 4)},
        "kernel_time": per_op,
        "tree_step": tree,
        "full_layer_step": {"us": round(full_us, 1), "hbm_frac": round(step_bytes / (full_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
        "sample_accept": {"us": round(accept_us, 1), "temperature": 0.8, "gamma": gamma, "vocab": V, "dtype": "f64",
                          "logit_bytes": (2 * gamma + 1) * V * 4},
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity_sample"] = cpu_baseline(args, cfg, weights, kpre, vpre, bounds, ctx, ctx_len, dev)
    print(json.dumps(out), flush=True)
    es.easyspec_destroy(ctx)


def cpu_baseline(args, cfg, weights, kpre, vpre, bounds, ctx, ctx_len, dev):
    """The oracle, as it stands, on the host cores: fuzzy draft steps at the same context on the
    same weights and KV prefix; the first step doubles as a full-size parity sample."""
    import torch
    import easyspec_synth as synth
    import paper_2502_02493_amd as es
    from oracle import easyspec_oracle as eso

    cores = int(os.environ.get("OMP_NUM_THREADS", 0)) or (os.cpu_count() or 1)
    model = eso.Model(cfg, weights, ctx_len + 64)
    seq = eso.Sequence(model)
    seq.import_kv(kpre, vpre)
    tok = int(synth.make_tokens(args.seed + 4, 1, cfg["vocab"])[0])

    es.easyspec_truncate(ctx, 0, ctx_len)
    tin = torch.tensor([tok], dtype=torch.int32, device=dev)
    tout = torch.zeros(1, dtype=torch.int32, device=dev)
    lg = torch.zeros(1, cfg["vocab"], dtype=torch.float32, device=dev)
    es.easyspec_draft_step(ctx, tin, tout, lg)
    torch.cuda.synchronize()
    got = lg[0].cpu().numpy().astype(np.float64)

    t0 = time.perf_counter()
    want = seq.fuzzy_step(bounds, tok)
    n, tk = 1, tok
    while time.perf_counter() - t0 < args.cpu_seconds and n < 64:
        tk = eso.argmax(seq.fuzzy_step(bounds, tk))
        n += 1
    dt = time.perf_counter() - t0
    wid, margin = eso.argmax(want, with_margin=True)
    parity = {"what": "one fuzzy draft step at full size, logits vs oracle",
              "rel_l2": float(np.linalg.norm(got - want) / np.linalg.norm(want)),
              "argmax_equal": bool(int(tout.item()) == wid), "oracle_top2_margin_over_std": float(margin / np.std(want))}
    base = {"value": round(n / dt, 4), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{n} fuzzy draft steps (batch 1, context {ctx_len}+) in {dt:.1f}s on the same weights and KV prefix"}
    return base, parity


if __name__ == "__main__":
    main()
