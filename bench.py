#!/usr/bin/env python3
"""Benchmark of the LVSpec verify-step hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input, through the C ABI:
    layers x lvspec_verify_attn  ->  lvspec_visual_relevance  ->  lvspec_loose_accept
Inputs are seeded, synthetic and resident in HBM before the timed region starts.  The headline
workload is the 64-layer stack of the Qwen2.5-VL-32B shape with five draft tokens (the
configuration the metric "verify-step latency" is quoted on): 64 distinct seeded KV caches
(4.3 GB) are streamed per step, so every attention call reads cold data.  Single-layer workloads
(c1, c2, c3) rotate over more than 1 GB of distinct KV caches for the same reason.

Prints ONE JSON line: throughput of the headline step, per-entry-point rooflines against the HBM
peak, the other configurations under "workloads" (same protocol, fewer steps), the headline step
replayed from a captured HIP graph, and the CPU oracle timed on one full headline step.
Timing protocol: W untimed steps, then K steps between two synchronisations (ms_per_step is
their mean on the host clock); every step is also bracketed by HIP events on the launch
stream, and "median"/"min" are taken over those K repetitions.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import subprocess
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E peak
# kernels one call of each entry point launches; the durations in `rooflines` are per call
KERNELS_OF = {
    "verify_attn": "lvspec_verify_attn = attn_split_kernel + attn_combine_kernel",
    "visual_relevance": ("lvspec_visual_relevance = gemm_stream_kernel<REL> + rel_cand_kernel + "
                         "rel_merge_kernel"),
    "lm_head_accept": ("lvspec_loose_accept = gemm_stream_kernel<LMH> + accept_finalize_kernel + "
                       "accept_decide_kernel"),
}
# the configurations timed besides the headline (name, draft rows override, steps)
EXTRA_WORKLOADS = [("c1", 0), ("c2", 0), ("c3", 0), ("c4", 3), ("c4", 8), ("c4t", 0), ("c5", 0)]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4",
                    choices=["c1", "c2", "c3", "c4", "c5", "c1t", "c2t", "c4t"],
                    help="headline workload.  c1..c5: the chain-draft configurations; c?t: the "
                         "same shapes with a draft tree of two chains of ten (c1t: four) tokens")
    ap.add_argument("--gamma", type=int, default=0, help="override the number of draft rows")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", action="store_true",
                    help="time the headline workload only (no other configurations, no graph "
                         "replay): what the profiling runs use")
    ap.add_argument("--prepared-norms", action="store_true",
                    help="hand lvspec_visual_relevance the inverse norms of lvspec_hv_prepare "
                         "(computed once, outside the timed region, as at prefill)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one plain elementwise kernel that reads 1 GiB and writes "
                         "1 GiB (reference point for HBM byte counters under rocprofv3 --pmc)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="HBM bytes and matrix-core use per launch from rocprofv3 counter runs "
                         "(see profiles/README.md for how it is made)")
    return ap.parse_args()


def resolve(name, gamma, layers, L, synth):
    cfg = synth.CONFIGS[name]
    if gamma:
        if cfg.n_branches > 1:
            sys.exit("bench.py: --gamma applies to the chain-draft workloads only")
        cfg = cfg.with_(gamma=gamma, pst_window=gamma, n_loose=L.n_loose(cfg.lam, gamma))
    if layers:
        cfg = cfg.with_(layers=layers)
    return cfg


class Workload:
    """Inputs of one configuration resident in HBM and the argument blocks of its calls."""

    def __init__(self, cfg, L, synth, dev, prepared_norms=False):
        self.cfg, self.L, self.synth, self.dev = cfg, L, synth, dev
        lib = self.lib = L.raw()
        self.layer_bytes = cfg.kv_bytes_per_layer
        if cfg.layers > 1:
            self.n_kv = cfg.layers
        else:
            self.n_kv = min(64, max(2, int(np.ceil(1.2e9 / self.layer_bytes))))   # cold rotation
        self.kv_sets = [synth.attn_inputs(cfg, layer=l, device=dev) for l in range(self.n_kv)]
        s0 = self.kv_sets[0]
        kv_len = torch.from_numpy(s0["kv_len"]).to(dev)
        vis_b = torch.from_numpy(s0["vis_begin"]).to(dev)
        vis_e = torch.from_numpy(s0["vis_end"]).to(dev)
        self.hv_bytes = cfg.B * cfg.vis_len * cfg.d * 2
        self.n_hv = 1 if cfg.layers > 1 else max(1, min(8, int(np.ceil(6e8 / self.hv_bytes))))
        self.hid = [synth.hidden_inputs(cfg.with_(seed=cfg.seed + 1000 * r), "literal", device=dev)
                    for r in range(self.n_hv)]
        l_v = torch.from_numpy(self.hid[0]["l_v"]).to(dev)
        self.w = synth.lm_head(cfg, device=dev)
        # a draft tree stores the rows of its chains one after the other: attention and relevance
        # see gamma rows per sequence, the accept call B * n_branches chains of chain_len rows
        self.n_br, self.K = cfg.n_branches, cfg.chain_len
        self.chains = cfg.B * self.n_br
        self.tree_mask = cfg.tree_mask()
        self.draft = torch.from_numpy(synth.draft_ids_uniform(cfg)).to(dev).reshape(self.chains,
                                                                                    self.K)
        out = torch.empty((cfg.B, cfg.gamma, cfg.Hq, cfg.D), dtype=torch.bfloat16, device=dev)
        self.rel = torch.empty((cfg.B, cfg.gamma), dtype=torch.float32, device=dev)
        acc_outs = L.alloc_accept_outputs(self.chains, self.K, cfg.V, 4, dev, n_branches=self.n_br)
        self.keep = [kv_len, vis_b, vis_e, l_v, out, acc_outs]

        self.attn_args = []
        for s in self.kv_sets:
            self.attn_args.append(L.verify_attn_args(
                s["q"], s["k"], s["v"], kv_len, out=out, vis_begin=vis_b, vis_end=vis_e,
                max_kv_len=max(cfg.kv_len), kv_len_host=list(cfg.kv_len),
                draft_mask=self.tree_mask))
        ws = torch.empty((max(256, lib.lvspec_verify_attn_workspace(C.byref(self.attn_args[0]))),),
                         dtype=torch.uint8, device=dev)
        for a in self.attn_args:
            a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
        self.keep.append(ws)
        self.rel_args = []
        for h in self.hid:
            inv = L.hv_prepare(h["h_v"]) if prepared_norms else None    # once, as at prefill
            self.keep.append(inv)
            self.rel_args.append(L.visual_relevance_args(h["h_d"], h["h_v"], l_v, cfg.top_n,
                                                         relevance=self.rel, hv_inv_norm=inv))
        ws = torch.empty((max(256, lib.lvspec_visual_relevance_workspace(
            C.byref(self.rel_args[0]))),), dtype=torch.uint8, device=dev)
        for a in self.rel_args:
            a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
        self.keep.append(ws)
        self.acc_args = L.loose_accept_args(
            self.hid[0]["h_d"].reshape(self.chains, self.K, cfg.d), self.w, self.draft,
            self.rel.reshape(self.chains, self.K), cfg.n_loose, cfg.pst_window, topk=4,
            loose_topk_gate=0, outs=acc_outs, n_branches=self.n_br)
        ws = torch.empty((max(256, lib.lvspec_loose_accept_workspace(C.byref(self.acc_args))),),
                         dtype=torch.uint8, device=dev)
        self.acc_args.workspace, self.acc_args.workspace_bytes = ws.data_ptr(), ws.numel()
        self.keep.append(ws)
        self.plan = L.describe_plan(attn=self.attn_args[0], rel=self.rel_args[0],
                                    accept=self.acc_args)
        # algorithmic bytes: every K/V row once, Q and O once (per layer); H_V + H_D once;
        # lm_head + H_D once
        self.alg_bytes = {
            "verify_attn": self.layer_bytes + 2 * cfg.B * cfg.gamma * cfg.Hq * cfg.D * 2,
            "visual_relevance": self.hv_bytes + cfg.B * cfg.gamma * cfg.d * 2,
            "lm_head_accept": cfg.V * cfg.d * 2 + cfg.B * cfg.gamma * cfg.d * 2,
        }

    def check(self, rc):
        if rc != 0:
            raise self.L.LvspecError(rc)

    def run_step(self, step, stream, events=None):
        lib, sp, layers = self.lib, stream.cuda_stream, self.cfg.layers
        if events:
            events[0].record(stream)
        if layers > 1:
            for l in range(layers):
                self.check(lib.lvspec_verify_attn(C.byref(self.attn_args[l]), sp))
        else:
            self.check(lib.lvspec_verify_attn(C.byref(self.attn_args[step % self.n_kv]), sp))
        if events:
            events[1].record(stream)
        self.check(lib.lvspec_visual_relevance(C.byref(self.rel_args[step % self.n_hv]), sp))
        if events:
            events[2].record(stream)
        self.check(lib.lvspec_loose_accept(C.byref(self.acc_args), sp))
        if events:
            events[3].record(stream)

    def time(self, steps, warmup):
        """W untimed steps, K timed ones; per-step HIP events on the launch stream."""
        stream = torch.cuda.current_stream()
        for s in range(warmup):
            self.run_step(s, stream)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            self.run_step(s, stream, evs[s])
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        layers = self.cfg.layers
        per = {"verify_attn": np.array([e[0].elapsed_time(e[1]) for e in evs]) * 1e3 / layers,
               "visual_relevance": np.array([e[1].elapsed_time(e[2]) for e in evs]) * 1e3,
               "lm_head_accept": np.array([e[2].elapsed_time(e[3]) for e in evs]) * 1e3}
        step_ms = np.array([e[0].elapsed_time(e[3]) for e in evs])
        return wall_ms, step_ms, per

    def time_attn_series(self, reps=5):
        """lvspec_verify_attn alone, back to back over the cold rotation (what a stack of
        layers of this shape costs per layer): median and min over `reps` series."""
        stream = torch.cuda.current_stream()
        sp, n = stream.cuda_stream, 2 * self.n_kv
        out = []
        for r in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for i in range(n):
                self.check(self.lib.lvspec_verify_attn(C.byref(self.attn_args[i % self.n_kv]), sp))
            e1.record(stream)
            torch.cuda.synchronize()
            if r > 0:                       # the first series warms up
                out.append(e0.elapsed_time(e1) * 1e3 / n)
        return float(np.median(out)), float(min(out))

    def time_graph(self, steps):
        """The same step captured once into a HIP graph and replayed."""
        stream = torch.cuda.current_stream()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                self.run_step(0, side)
        torch.cuda.synchronize()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        reps = []
        for _ in range(steps):
            t0 = time.perf_counter()
            g.replay()
            torch.cuda.synchronize()
            reps.append((time.perf_counter() - t0) * 1e3)
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, float(np.median(reps)), float(min(reps))

    def roofs(self, per, counters):
        out = {}
        for key, us in per.items():
            med = float(np.median(us))
            gbs = self.alg_bytes[key] / (float(us.mean()) * 1e-6) / 1e9
            c = counters.get(key, {})
            # mfma_frac_of_peak: executed bf16 MFMA flops of the streaming kernel over its
            # duration, as a fraction of the 2.5 PFLOP/s dense peak (rocprofv3 counters)
            out[key] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                        "traffic": c.get("traffic"), "algorithmic_bytes": int(self.alg_bytes[key]),
                        "avg_us": round(float(us.mean()), 2), "median_us": round(med, 2),
                        "min_us": round(float(us.min()), 2),
                        "mfma_frac_of_peak": c.get("mfma_frac_of_peak")}
        return out

    def config(self):
        cfg = self.cfg
        return {"workload": cfg.name, "B": cfg.B, "gamma": cfg.gamma, "Hq": cfg.Hq,
                "Hkv": cfg.Hkv, "D": cfg.D, "kv_len": list(cfg.kv_len), "layers": cfg.layers,
                "visual_tokens": cfg.vis_len, "hidden": cfg.d, "vocab": cfg.V,
                "top_n": cfg.top_n, "n_loose": cfg.n_loose, "pst_window": cfg.pst_window,
                "draft_tree_branches": self.n_br, "chain_len": self.K,
                "distinct_kv_caches": self.n_kv}


def load_counters(path, wl, lib_version):
    """HBM bytes and matrix-core use per launch, replayed from the tracked counter summary.  The
    file is stamped with the library version, the commit and the launch plan it was taken at;
    figures are handed on only when version and plan still match this run, else they are null."""
    info = {"file": os.path.relpath(path, ROOT), "replayed": True, "commit": None, "match": False}
    try:
        data = json.load(open(path))
    except (OSError, ValueError) as e:
        info["error"] = f"{type(e).__name__}: {e}"
        return {}, info
    stamp = data.get("stamp", {})
    info["commit"] = stamp.get("commit")
    plans = stamp.get("plans", {})
    name = wl.cfg.name
    if stamp.get("library_version") != lib_version or plans.get(name) != wl.plan:
        return {}, info
    info["match"] = True
    out = {}
    for key in ("verify_attn", "visual_relevance", "lm_head_accept"):
        out[key] = {"traffic": data.get(name, {}).get(key),
                    "mfma_frac_of_peak": data.get(name + ":mfma", {}).get(key, {}).get(
                        "frac_of_bf16_peak")}
    return out, info


def cpu_baseline(wl):
    """One full step of the oracle, as it stands, on the host cores of this machine."""
    import oracle
    cfg, synth = wl.cfg, wl.synth
    t_attn = 0.0
    for l in range(cfg.layers):
        s = wl.kv_sets[l % wl.n_kv]
        qh, kh, vh = (synth.from_torch_bf16(s[x]) for x in ("q", "k", "v"))
        t = time.perf_counter()
        oracle.verify_attn(qh, kh, vh, s["kv_len"], s["vis_begin"], s["vis_end"],
                           draft_mask=wl.tree_mask)
        t_attn += time.perf_counter() - t
    hd_h = synth.from_torch_bf16(wl.hid[0]["h_d"])
    hv_h = synth.from_torch_bf16(wl.hid[0]["h_v"])
    t = time.perf_counter()
    rel_o = oracle.visual_relevance(hd_h, hv_h, wl.hid[0]["l_v"], cfg.top_n)
    t_rel = time.perf_counter() - t
    w_h = synth.from_torch_bf16(wl.w)
    t = time.perf_counter()
    oracle.loose_accept(hd_h.reshape(wl.chains, wl.K, cfg.d), w_h, wl.draft.cpu().numpy(),
                        rel_o.astype(np.float32).reshape(wl.chains, wl.K), cfg.n_loose,
                        cfg.pst_window, topk=4, n_branches=wl.n_br)
    t_acc = time.perf_counter() - t
    step_s = t_attn + t_rel + t_acc
    return {"value": round(cfg.B * cfg.gamma / step_s, 3), "unit": "tokens/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": (f"one full step of {cfg.name}: {cfg.layers} attention layer(s), relevance "
                       f"over {cfg.vis_len} video rows, lm_head + accept over {cfg.V} vocabulary "
                       "rows; nothing scaled"),
            "step_seconds": round(step_s, 3),
            "seconds": {"verify_attn": round(t_attn, 3), "visual_relevance": round(t_rel, 3),
                        "lm_head_accept": round(t_acc, 3)}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        sys.exit(2)
    from paper_2604_05650_amd import binding as L
    from paper_2604_05650_amd import synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = resolve(args.workload, args.gamma, args.layers, L, synth)
    wl = Workload(cfg, L, synth, dev, prepared_norms=args.prepared_norms)

    if args.calibrate_copy:
        src = torch.zeros((1 << 28,), dtype=torch.int32, device=dev)       # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)          # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ headline, timed
    wall_ms, step_ms, per = wl.time(args.steps, args.warmup)
    counters, counter_info = load_counters(args.traffic_json, wl, L.version())
    roofs = wl.roofs(per, counters)
    layers = cfg.layers
    tot = {k: float(np.median(v)) * (layers if k == "verify_attn" else 1) for k, v in per.items()}
    dominant = max(tot, key=tot.get)
    tokens = cfg.B * cfg.gamma

    graph = None
    if not args.only:
        g_mean, g_med, g_min = wl.time_graph(max(5, args.steps // 2))
        graph = {"ms_per_step": round(g_mean, 4), "median_ms_single_replay": round(g_med, 4),
                 "min_ms_single_replay": round(g_min, 4)}

    cpu = None if args.no_cpu_baseline else cpu_baseline(wl)
    head_cfg, head_plan = wl.config(), wl.plan
    del wl
    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ the other configurations
    others = {}
    if not args.only:
        for name, gam in EXTRA_WORKLOADS:
            c = resolve(name, gam, 0, L, synth)
            if c == cfg:
                continue
            w2 = Workload(c, L, synth, dev, prepared_norms=args.prepared_norms)
            k = max(5, min(args.steps, 12 if c.layers > 1 or c.B > 1 else 20))
            wm, sm, p2 = w2.time(k, 3)
            cn, _ = load_counters(args.traffic_json, w2, L.version())
            r2 = w2.roofs(p2, cn)
            if c.layers == 1:
                # a single-layer step times its one attention call right behind the previous
                # step's last small kernel; the same call in a series is the per-layer cost
                med, mn = w2.time_attn_series()
                r2["verify_attn"]["back_to_back_median_us"] = round(med, 2)
                r2["verify_attn"]["back_to_back_min_us"] = round(mn, 2)
                r2["verify_attn"]["back_to_back_frac"] = round(
                    w2.alg_bytes["verify_attn"] / (med * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
            label = name + (f"-gamma{gam}" if gam else "")
            others[label] = {
                "config": w2.config(), "plan": w2.plan, "steps": k, "ms_per_step": round(wm, 4),
                "median_ms": round(float(np.median(sm)), 4), "min_ms": round(float(sm.min()), 4),
                "tokens_per_s": round(c.B * c.gamma / (wm * 1e-3), 1),
                "rooflines": {e: {f: r2[e][f] for f in r2[e]
                                  if f in ("median_us", "min_us", "frac", "traffic") or
                                  f.startswith("back_to_back")} for e in r2}}
            del w2
            torch.cuda.empty_cache()

    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"],
                                capture_output=True, text=True, timeout=10).stdout.strip() or None
    except (OSError, subprocess.SubprocessError):
        commit = None
    commit = commit or os.environ.get("LVSPEC_COMMIT") or None

    res = {
        "metric": "draft tokens verified per second (whole verify step: layers x verify attention "
                  "+ visual relevance + lm_head/loose accept)",
        "value": round(tokens / (wall_ms * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4),
        "verify_step_latency_us": round(wall_ms * 1e3, 1),
        "timing": {"repetitions": args.steps, "median_ms": round(float(np.median(step_ms)), 4),
                   "min_ms": round(float(step_ms.min()), 4),
                   "what": "per-step HIP events on the launch stream, first call to last kernel"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": head_cfg,
        "plan": head_plan,
        "library_version": L.version(),
        "roofline": dict(roofs[dominant], kernel=KERNELS_OF[dominant]),
        "rooflines": roofs,
        "counters": counter_info,
        "breakdown_us": {"verify_attn_per_layer": roofs["verify_attn"]["median_us"],
                         "verify_attn_per_layer_min": roofs["verify_attn"]["min_us"],
                         "visual_relevance": roofs["visual_relevance"]["median_us"],
                         "lm_head_accept": roofs["lm_head_accept"]["median_us"],
                         "gpu_step_ms_events": round(float(np.median(step_ms)), 4)},
        "graph_replay": graph,
        "graph_replay_ms_per_step": None if graph is None else graph["ms_per_step"],
        "workloads": others,
        "relevance_norms": "prepared" if args.prepared_norms else "in-pass",
        "commit": commit,
        "cpu_baseline": cpu,
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
