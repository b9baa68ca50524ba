#!/usr/bin/env python3
"""Benchmark of the EasySpec draft hot path on one MI355X.

One "step" is one drafting iteration of the three-stage loop: bonus calibration over gamma+1
tokens (which also yields the first draft token), gamma-1 layer-parallel fuzzy draft steps,
and greedy acceptance against a synthetic verifier output.  `value` is drafted tokens per
second over whole iterations (gamma tokens per iteration and sequence); the per-call figures the
metric names (fuzzy draft-step tokens/s, calibration microseconds, each with its share of the HBM
roofline) are reported in the same JSON line, for the headline workload and, under `workloads`,
for every other configuration (calibration-dominant, long-context batch 4, Qwen2-7B shape at
three layer-parallel sizes) and, under `group_size_sweep`, for N = 1, 2, 4, 8 on the headline.

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
# WRITE_SIZE runs summarised in profiles/hbm_traffic_llama3_8b_ctx2048.md (scaled by a 1 GiB copy).  A
# committed figure, not a reading of the run it is printed in.
COMMITTED_TRAFFIC_KIB = {"llama3_8b_ctx2048": 230061.3}
OPS = ("qkv", "attn", "oproj", "gateup", "down", "head")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Env:
    """torch, the binding, the input generators, the device and the stream every call is ordered on."""

    def __init__(self):
        import torch
        import easyspec_synth as synth
        import paper_2502_02493_amd as es
        self.torch, self.synth, self.es = torch, synth, es
        self.dev = torch.device("cuda:0")
        self.stream = torch.cuda.current_stream().cuda_stream
        self.op_id = dict(qkv=es.EASYSPEC_OP_QKV, attn=es.EASYSPEC_OP_ATTN, oproj=es.EASYSPEC_OP_OPROJ,
                          gateup=es.EASYSPEC_OP_GATEUP, down=es.EASYSPEC_OP_DOWN, head=es.EASYSPEC_OP_HEAD)

    def events(self, n):
        return [self.torch.cuda.Event(enable_timing=True) for _ in range(n)]


def op_bytes(cfg, kv_bytes):
    """Algorithmic HBM bytes of each kernel class in one forward pass: its weights once (the KV slots read, for attention)."""
    e = 2 if cfg["dtype"] == "bf16" else 4
    L, d, F, V = cfg["n_layers"], cfg["d_model"], cfg["d_ffn"], cfg["vocab"]
    hq, rqkv = cfg["n_q_heads"] * cfg["head_dim"], (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"]
    return dict(qkv=L * rqkv * d * e, attn=int(kv_bytes), oproj=L * d * hq * e, gateup=L * 2 * F * d * e, down=L * F * d * e,
                head=V * d * e)


class Loop:
    """Drafting iterations of one context: calibration of the sequences' accepted tokens + bonus token, gamma-1
    fuzzy draft steps for all sequences at once, greedy acceptance; every iteration starts from the same
    prefix lengths (the fuzzy slots of the last one are dropped, as a calibration does)."""

    def __init__(self, env, ctx, cfg, ctx_lens, gamma, seed, draw_calib=False):
        torch, synth = env.torch, env.synth
        self.env, self.ctx, self.cfg, self.ctx_lens, self.gamma = env, ctx, cfg, list(ctx_lens), gamma
        self.B, self.M = len(ctx_lens), gamma + 1
        B = self.B
        self.calib_tok = torch.from_numpy(synth.make_tokens(seed + 2, B * 16, cfg["vocab"]).reshape(B, 16)).to(env.dev)
        self.n_tok = np.full(B, self.M, np.int32)
        self.draft = torch.zeros(gamma + 1, B, dtype=torch.int32, device=env.dev)       # draft[j][b] = j-th drafted token of b
        self.target = torch.from_numpy(synth.make_tokens(seed + 3, B * (gamma + 1), cfg["vocab"]).reshape(B, gamma + 1)).to(env.dev)
        self.acc = torch.zeros(B, dtype=torch.int32, device=env.dev)
        self.bonus = torch.zeros(B, dtype=torch.int32, device=env.dev)
        # Calibration length: gamma + 1 tokens (every drafted token accepted, the costliest case), or, for the
        # calibration-dominant workload, accepted-length + 1 with the accepted length drawn uniformly from
        # 0 .. gamma by the seeded generator (partial rewrites of the fuzzy slots).
        self.draw_calib = draw_calib
        self.rng = np.random.Generator(np.random.Philox(key=[seed, 77]))
        self.calib_lens = []

    def reset(self):
        for b, n in enumerate(self.ctx_lens):
            self.env.es.easyspec_truncate(self.ctx, b, n)

    def calibrate(self, record=False):
        self.reset()
        if self.draw_calib:
            self.n_tok[:] = self.rng.integers(1, self.M + 1, size=self.B)
        if record:
            self.calib_lens.append(float(np.mean(self.n_tok)))
        self.env.es.easyspec_calibrate(self.ctx, self.calib_tok, self.n_tok, self.draft[0], None, 0)   # first draft token -> draft[0]

    def steps(self):
        for j in range(1, self.gamma):
            self.env.es.easyspec_draft_step(self.ctx, self.draft[j - 1], self.draft[j], None)

    def accept(self):
        es = self.env.es
        d = self.draft[: self.gamma] if self.B == 1 else self.draft[: self.gamma].t().contiguous()   # [B][gamma]
        es.easyspec_greedy_accept(d, self.target, self.B, self.gamma, self.acc, self.bonus, self.env.stream)

    def iteration(self):
        self.calibrate()
        self.steps()
        self.accept()

    def run_wall(self, steps, warmup):
        """Whole iterations, no events inside the timed region.  Returns seconds per iteration."""
        torch = self.env.torch
        for _ in range(warmup):
            self.iteration()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.iteration()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def run_split(self, steps):
        """The same iterations with stream events between the stages.  Returns (calibration us, draft-step us)."""
        evs = [self.env.events(3) for _ in range(steps)]
        for ev in evs:
            self.reset()
            ev[0].record()
            self.calibrate(record=True)
            ev[1].record()
            self.steps()
            ev[2].record()
            self.accept()
        self.env.torch.cuda.synchronize()
        calib_us = 1e3 * float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
        step_us = 1e3 * float(np.mean([e[1].elapsed_time(e[2]) for e in evs])) / (self.gamma - 1)
        return calib_us, step_us

    def bytes(self):
        """Algorithmic bytes of one draft step and of one calibration (weights once + the KV slots read)."""
        cfg = self.cfg
        self.reset()
        step_bytes = int(self.env.es.easyspec_step_bytes(self.ctx))
        e = 2 if cfg["dtype"] == "bf16" else 4
        m_mean = float(np.mean(self.calib_lens)) if self.calib_lens else float(self.M)
        slot = cfg["n_layers"] * 2 * cfg["n_kv_heads"] * cfg["head_dim"] * e
        return step_bytes, int(step_bytes + self.B * (m_mean - 1) * slot), m_mean

    def report(self, steps, warmup):
        sec = self.run_wall(steps, warmup)
        calib_us, step_us = self.run_split(steps)
        step_bytes, calib_bytes, m_mean = self.bytes()
        return sec, {
            "tokens_per_s": round(self.B * self.gamma / sec, 2), "ms_per_iteration": round(1e3 * sec, 4),
            "draft_step": {"us": round(step_us, 1), "tokens_per_s": round(self.B * 1e6 / step_us, 2), "bytes": step_bytes,
                           "hbm_frac": round(step_bytes / (step_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
            "calibrate": {"us": round(calib_us, 1), "tokens": self.M if not self.draw_calib else round(m_mean, 2),
                          "tokens_drawn": "uniform 1..%d" % self.M if self.draw_calib else "fixed", "bytes": calib_bytes,
                          "hbm_frac": round(calib_bytes / (calib_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}}

    def timed(self, what, reps):
        """Every kernel of `reps` x (the draft steps of an iteration | a calibration) with a start and a stop event
        bound to its dispatch, as a kernel trace times them.  Returns (microseconds per launch, kernel class per
        launch, calls): calls = draft steps or calibrations covered."""
        es = self.env.es
        cap = reps * 4096
        ms, op = np.zeros(cap, np.float32), np.zeros(cap, np.int32)
        us_all, op_all = [], []
        for _ in range(reps):
            if what == "step":
                self.calibrate()
            else:
                self.reset()
            es.easyspec_profile_begin(self.ctx, es.EASYSPEC_OP_ALL, 4096)
            if what == "step":
                self.steps()
            else:
                self.calibrate()
            n, _ = es.easyspec_profile_end(self.ctx, ms, op)
            us_all.append(1e3 * ms[:n].astype(np.float64))
            op_all.append(op[:n].copy())
        return np.concatenate(us_all), np.concatenate(op_all), reps * ((self.gamma - 1) if what == "step" else 1)

    def kernel_table(self, reps=3):
        """Per kernel class: launches, microseconds (each kernel's own begin-to-end time) and algorithmic bytes per
        draft step and per calibration, with the share of the HBM roofline; and how the kernels' durations add up
        against the duration of the whole call (dependent kernels run back to back)."""
        env = self.env
        step_bytes, _, _ = self.bytes()
        weights = op_bytes(self.cfg, 0)
        per = op_bytes(self.cfg, step_bytes - sum(weights.values()))
        table = {name: {} for name in OPS}
        for what, key in (("step", "per_step"), ("calibration", "per_calibration")):
            us, op, calls = self.timed(what, reps)
            for name in OPS:
                sel = op == env.op_id[name]
                t = float(us[sel].sum()) / calls
                table[name][key] = {"launches": round(int(sel.sum()) / calls, 1), "us": round(t, 1), "bytes": per[name],
                                    "hbm_frac": round(per[name] / (t * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
            table["all_kernels_" + key] = {"launches": round(len(us) / calls, 1), "sum_us": round(float(us.sum()) / calls, 1)}
        return table


def device_kv_prefix(env, ctx, cfg, ctx_lens, seed):
    """KV prefixes drawn on the device (N(0,1) in the storage type): for timing, where only their size matters."""
    torch = env.torch
    gen = torch.Generator(device=env.dev).manual_seed(seed)
    L, hkv, hd = cfg["n_layers"], cfg["n_kv_heads"], cfg["head_dim"]
    for b, n in enumerate(ctx_lens):
        k = torch.randn(L, hkv, n, hd, device=env.dev, generator=gen).to(torch.bfloat16).view(torch.int16)
        v = torch.randn(L, hkv, n, hd, device=env.dev, generator=gen).to(torch.bfloat16).view(torch.int16)
        env.es.easyspec_kv_import(ctx, b, k, v, n)
        del k, v


def bounds_of(env, cfg, wl, N=None):
    es = env.es
    policy = es.EASYSPEC_POLICY_ALIGNED if wl["group_policy"] == "aligned" else es.EASYSPEC_POLICY_PACKED
    return es.easyspec_default_groups(cfg["n_layers"], N or wl["group_size"], policy)


def launches_per_step(bounds, n_layers):
    """Kernel launches of one fuzzy draft step at contexts long enough for split-KV attention."""
    return 1 + 4 * (len(bounds) - 1) + 2 * n_layers + 2      # embed; QKV, attention, merge, O per set; gate/up, down per layer; head, argmax


def other_workload(env, name, weights, steps, warmup, seed, sizes=None):
    """A configuration other than the headline: its own context (weights repacked from the same host arrays), device-drawn
    KV prefix, the same iteration loop.  sizes: layer-parallel sizes to run (default: the workload's own)."""
    synth, es = env.synth, env.es
    wl = dict(synth.WORKLOADS[name])
    cfg = synth.model_shape(wl["model"])
    ctx_lens = list(wl["context"]) if isinstance(wl["context"], tuple) else [wl["context"]]
    gamma = wl["gamma"]
    t0 = time.time()
    ctx = es.easyspec_create(es.make_config(cfg, len(ctx_lens), max(ctx_lens) + gamma + 16, 16), env.stream)
    out = {}
    try:
        es.easyspec_load_weights(ctx, weights)
        device_kv_prefix(env, ctx, cfg, ctx_lens, seed)
        for N in sizes or [wl["group_size"]]:
            bounds = bounds_of(env, cfg, wl, N)
            es.easyspec_set_groups(ctx, bounds)
            loop = Loop(env, ctx, cfg, ctx_lens, gamma, seed, draw_calib=wl.get("calib_tokens") == "uniform")
            _, rep = loop.report(steps, warmup)
            rep["config"] = {"shape": wl["model"], "contexts": ctx_lens, "batch": len(ctx_lens), "group_size": N, "gamma": gamma,
                             "sets": len(bounds) - 1, "launches_per_step": launches_per_step(bounds, cfg["n_layers"])}
            out[f"N={N}"] = rep
    finally:
        es.easyspec_destroy(ctx)
    log(f"[bench] workload {name} in {time.time() - t0:.1f}s")
    return out if sizes else out[f"N={wl['group_size']}"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama3_8b_ctx2048")
    ap.add_argument("--seed", type=int, default=2025)
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging; makes the result invalid)")
    ap.add_argument("--group-size", type=int, default=0, help="override the workload's layer-parallel size N (1 = sequential)")
    ap.add_argument("--no-extras", action="store_true",
                    help="the headline workload only: no tree levels, ablation, other workloads, sweep or CPU baseline (profiling runs)")
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
    if not torch.cuda.is_available():
        print("bench.py: no HIP device visible", file=sys.stderr)
        sys.exit(3)
    env = Env()
    synth, es = env.synth, env.es
    es.load_library()
    wl = dict(synth.WORKLOADS[args.workload])
    default_run = args.workload == "llama3_8b_ctx2048" and not args.layers and not args.group_size
    over = {"n_layers": args.layers} if args.layers else {}
    if args.group_size:
        wl["group_size"] = args.group_size
    cfg = synth.model_shape(wl["model"], **over)
    ctx_lens = list(wl["context"]) if isinstance(wl["context"], tuple) else [wl["context"]]
    gamma, B = wl["gamma"], len(ctx_lens)
    M = gamma + 1
    bounds = bounds_of(env, cfg, wl)
    max_ctx = max(ctx_lens) + M + max(gamma, 4 * 12) + 8      # room for the chain and for the widest tree timed below

    t0 = time.time()
    weights = synth.make_weights(cfg, args.seed)
    kpre = vpre = None
    if B == 1:
        kpre, vpre = synth.make_kv_prefix(cfg, args.seed + 1, ctx_lens[0])
    log(f"[bench] synthetic inputs drawn in {time.time() - t0:.1f}s")

    dev, stream = env.dev, env.stream
    ctx = es.easyspec_create(es.make_config(cfg, B, max_ctx, 16), stream)
    t0 = time.time()
    es.easyspec_load_weights(ctx, weights)
    es.easyspec_set_groups(ctx, bounds)
    if B == 1:
        es.easyspec_kv_import(ctx, 0, kpre, vpre, ctx_lens[0])
    else:
        device_kv_prefix(env, ctx, cfg, ctx_lens, args.seed + 1)
    log(f"[bench] weights packed and KV prefix imported in {time.time() - t0:.1f}s")

    if args.copy_mib:
        src = torch.ones(args.copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads and writes copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst

    loop = Loop(env, ctx, cfg, ctx_lens, gamma, args.seed, draw_calib=wl.get("calib_tokens") == "uniform")
    sec, head = loop.report(args.steps, args.warmup)
    step_bytes, calib_bytes, m_mean = loop.bytes()
    e = 2 if cfg["dtype"] == "bf16" else 4
    gu_bytes = 2 * cfg["d_ffn"] * cfg["d_model"] * e

    # Dominant kernel (gate/up projection: 2*F*d weights per launch): the same iterations again with a start and a
    # stop event bound to every kernel's dispatch (what a kernel trace does); its launches are those of class GATEUP.
    per_iter = 4096
    ms, op = np.zeros(per_iter, np.float32), np.zeros(per_iter, np.int32)
    gu_us = []
    for _ in range(args.steps):
        es.easyspec_profile_begin(ctx, es.EASYSPEC_OP_ALL, per_iter)
        loop.iteration()
        n, _ = es.easyspec_profile_end(ctx, ms, op)
        gu_us.append(1e3 * ms[:n][op[:n] == es.EASYSPEC_OP_GATEUP].astype(np.float64))
    gu_us = np.concatenate(gu_us)
    n_timed = int(gu_us.size)
    gu_ms = 1e-3 * float(gu_us.mean())
    gu_gbs = gu_bytes / (gu_ms * 1e-3) / 1e9
    kernels = loop.kernel_table()

    # what a kernel that only reads reaches on this device (same loads as the weight stream), 4 GiB per pass
    probe = torch.empty(1 << 30, dtype=torch.int32, device=dev)
    probe.zero_()
    sink = torch.empty(es.easyspec_stream_read_sink_floats(), dtype=torch.float32, device=dev)
    pe = env.events(2)
    for k in range(8):
        if k == 3: pe[0].record()
        es.easyspec_stream_read(probe, probe.numel() * 4, sink, stream)
    pe[1].record()
    torch.cuda.synchronize()
    stream_gbs = 5 * probe.numel() * 4 / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e9
    del probe

    traffic_kib = args.traffic_kib if args.traffic_kib is not None else (COMMITTED_TRAFFIC_KIB.get(args.workload) if default_run else None)
    head["draft_step"]["frac_of_stream_read"] = round(step_bytes / (head["draft_step"]["us"] * 1e-6) / 1e9 / stream_gbs, 4)
    out = {
        "metric": "draft tokens/sec (whole drafting iteration: calibration + fuzzy steps + accept)",
        "value": round(B * gamma / sec, 2),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * sec, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload + ("" if not args.layers else f"_L{args.layers}_INVALID"),
                   "shape": cfg["name"], "context": ctx_lens[0] if B == 1 else ctx_lens, "batch": B,
                   "group_size": wl["group_size"], "sets": [int(x) for x in bounds], "gamma": gamma, "calib_tokens": M,
                   "launches_per_step": launches_per_step(bounds, cfg["n_layers"])},
        "draft_step": head["draft_step"],
        "calibrate": head["calibrate"],
        "roofline": {"bound": "hbm", "kernel": "gateup_kernel", "achieved": round(gu_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gu_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic_kib * 1024 if traffic_kib else None,
                     "traffic_source": "profiles/hbm_traffic_llama3_8b_ctx2048.md (rocprofv3 --pmc runs of this workload; a committed figure, not a reading of this run)" if traffic_kib else None,
                     "bytes_per_launch": int(gu_bytes), "avg_launch_us": round(1e3 * gu_ms, 2),
                     "median_launch_us": round(float(np.median(gu_us)), 2), "min_launch_us": round(float(gu_us.min()), 2),
                     "timing": "a start and a stop HIP event bound to the dispatch of every kernel of the timed iterations "
                               "(calibrations and draft steps), as a kernel trace times them; no correction applied; "
                               "profiles/kernel_stats_llama3_8b_ctx2048.md holds the rocprofv3 kernel trace of the same command",
                     "launches_timed": n_timed, "stream_read_gbs": round(stream_gbs, 1),
                     "frac_of_stream_read": round(gu_gbs / stream_gbs, 4)},
        "kernels": kernels,
    }
    if not args.no_extras and B == 1:
        out.update(extras(env, args, ctx, cfg, loop, step_bytes))
    if default_run and not args.no_extras:
        out["group_size_sweep"] = group_size_sweep(env, args, ctx, cfg, wl, ctx_lens)
    if not args.no_extras and not args.no_cpu_baseline and B == 1:
        es.easyspec_set_groups(ctx, bounds)
        out["cpu_baseline"], out["parity_sample"] = cpu_baseline(args, cfg, weights, kpre, vpre, bounds, ctx, ctx_lens[0], dev)
    elif "cpu_baseline" not in out:
        out["cpu_baseline"] = None
    es.easyspec_destroy(ctx)
    if default_run and not args.no_extras:
        del kpre, vpre
        n = max(6, args.steps // 3)
        w = {"llama3_8b_calib_ctx8192": other_workload(env, "llama3_8b_calib_ctx8192", weights, n, 2, args.seed + 10),
             "llama3_8b_batch4_long": other_workload(env, "llama3_8b_batch4_long", weights, n, 2, args.seed + 11)}
        del weights
        t0 = time.time()
        qw = synth.make_weights(synth.model_shape("qwen2_7b"), args.seed)
        log(f"[bench] Qwen2-7B-shaped weights drawn in {time.time() - t0:.1f}s")
        w["qwen2_7b_ctx4096"] = other_workload(env, "qwen2_7b_ctx4096", qw, n, 2, args.seed + 12, sizes=[2, 4, 7])
        out["workloads"] = w
    print(json.dumps(out), flush=True)


def extras(env, args, ctx, cfg, loop, step_bytes):
    """Beside the iteration, on the same context (not part of `value`): speculative-sampling acceptance, token-tree
    levels, the full-layer-parallel ablation."""
    torch, synth, es, dev, stream = env.torch, env.synth, env.es, env.dev, env.stream
    gamma, ctx_len = loop.gamma, loop.ctx_lens[0]
    n_tok = np.array([gamma + 1], np.int32)
    # acceptance by speculative sampling (temperature 0.8, the paper's second setting) on logits of this vocabulary
    V = cfg["vocab"]
    tl = torch.from_numpy(synth.make_logits(args.seed + 5, gamma + 1, V)).to(dev)
    dl = (tl[:gamma] + 0.7 * torch.from_numpy(synth.make_logits(args.seed + 6, gamma, V, std=1.0)).to(dev)).contiguous()
    ru = torch.from_numpy(synth.make_uniforms(args.seed + 7, gamma + 1)).to(dev)
    ws = torch.empty(es.easyspec_accept_workspace_bytes(1, gamma, V) // 8, dtype=torch.float64, device=dev)
    draft = loop.draft[:gamma].reshape(1, gamma).contiguous()
    sa = env.events(2)
    n_acc = 50
    for k in range(n_acc + 5):
        if k == 5: sa[0].record()
        es.easyspec_accept(draft, dl, tl, ru, ru[gamma:], 1, gamma, V, 0.8, loop.acc, loop.bonus, ws, stream)
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
        evs_t = env.events(2)
        reps = max(2, args.steps // 4)
        tot = 0.0
        for rep in range(reps + 1):
            es.easyspec_truncate(ctx, 0, ctx_len)
            es.easyspec_calibrate(ctx, loop.calib_tok, n_tok, loop.draft[0], None, 0)
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
    fl = env.events(2)
    reps = max(2, args.steps // 4)
    tot = 0.0
    for rep in range(reps + 1):
        loop.calibrate()
        fl[0].record()
        loop.steps()
        fl[1].record()
        torch.cuda.synchronize()
        if rep:
            tot += fl[0].elapsed_time(fl[1])
    full_us = 1e3 * tot / (reps * (gamma - 1))
    es.easyspec_set_parallel_mode(ctx, es.EASYSPEC_PARALLEL_ATTENTION)
    es.easyspec_truncate(ctx, 0, ctx_len)
    return {
        "tree_step": tree,
        "full_layer_step": {"us": round(full_us, 1), "hbm_frac": round(step_bytes / (full_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)},
        "sample_accept": {"us": round(accept_us, 1), "temperature": 0.8, "gamma": gamma, "vocab": V, "dtype": "f64",
                          "logit_bytes": (2 * gamma + 1) * V * 4}}


def group_size_sweep(env, args, ctx, cfg, wl, ctx_lens):
    """The headline workload at layer-parallel sizes 1 (sequential, Alg. 1), 2, 4 and 8: the paper's T_seq against T_fuzzy
    on one GPU, where the launch count stands in for its cross-GPU overlap."""
    es = env.es
    out = {}
    for N in (1, 2, 4, 8):
        b = bounds_of(env, cfg, wl, N)
        es.easyspec_set_groups(ctx, b)
        loop = Loop(env, ctx, cfg, ctx_lens, wl["gamma"], args.seed)
        for _ in range(2):
            loop.iteration()
        calib_us, step_us = loop.run_split(max(5, args.steps // 3))
        step_bytes, _, _ = loop.bytes()
        out[f"N={N}"] = {"sets": len(b) - 1, "launches_per_step": launches_per_step(b, cfg["n_layers"]), "draft_step_us": round(step_us, 1),
                         "hbm_frac": round(step_bytes / (step_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "calibrate_us": round(calib_us, 1)}
    es.easyspec_set_groups(ctx, bounds_of(env, cfg, wl))
    return out


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
              "max_abs_over_rms": float(np.max(np.abs(got - want)) / (np.linalg.norm(want) / np.sqrt(want.size))),
              "argmax_equal": bool(int(tout.item()) == wid), "oracle_top2_margin_over_std": float(margin / np.std(want))}
    base = {"value": round(n / dt, 4), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{n} fuzzy draft steps (batch 1, context {ctx_len}+) in {dt:.1f}s on the same weights and KV prefix"}
    return base, parity


if __name__ == "__main__":
    main()
