#!/usr/bin/env python3
"""Benchmark of the LVSpec verify-step hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input, through the C ABI:
    layers x lvspec_verify_attn  ->  lvspec_visual_relevance  ->  lvspec_loose_accept
Inputs are seeded, synthetic and resident in HBM before the timed region starts.  The default
workload is the 64-layer stack of the Qwen2.5-VL-32B shape (the configuration the metric
"verify-step latency" is quoted on): 64 distinct seeded KV caches (4.3 GB) are streamed per
step, so every attention call reads cold data.  Single-layer workloads (c1, c2, c3) rotate over
more than 1 GB of distinct KV caches for the same reason.

Prints ONE JSON line: throughput of the whole step, per-entry-point rooflines against the HBM peak,
and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5", "c1t", "c2t", "c4t"],
                    help="c1..c5: the chain-draft configurations; c?t: the same shapes with a "
                         "draft tree of two chains of ten (c1t: four) tokens")
    ap.add_argument("--gamma", type=int, default=0, help="override the number of draft rows")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a captured HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one plain elementwise kernel that reads 1 GiB and writes "
                         "1 GiB (reference point for HBM byte counters under rocprofv3 --pmc)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="measured HBM bytes per launch (written by profiles/README steps)")
    return ap.parse_args()


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
    cfg = synth.CONFIGS[args.workload]
    if args.gamma:
        if cfg.n_branches > 1:
            sys.exit("bench.py: --gamma applies to the chain-draft workloads only")
        cfg = cfg.with_(gamma=args.gamma, pst_window=args.gamma,
                        n_loose=L.n_loose(cfg.lam, args.gamma))
    if args.layers:
        cfg = cfg.with_(layers=args.layers)
    lib = L.raw()

    # ------------------------------------------------------------------ inputs (resident in HBM)
    layer_bytes = cfg.kv_bytes_per_layer
    if cfg.layers > 1:
        n_kv = cfg.layers
    else:
        n_kv = max(2, int(np.ceil(1.2e9 / layer_bytes)))      # cold-cache rotation
        n_kv = min(n_kv, 64)
    kv_sets = [synth.attn_inputs(cfg, layer=l, device=dev) for l in range(n_kv)]
    kv_len = torch.from_numpy(kv_sets[0]["kv_len"]).to(dev)
    vis_b = torch.from_numpy(kv_sets[0]["vis_begin"]).to(dev)
    vis_e = torch.from_numpy(kv_sets[0]["vis_end"]).to(dev)
    hv_bytes = cfg.B * cfg.vis_len * cfg.d * 2
    n_hv = 1 if cfg.layers > 1 else max(1, min(8, int(np.ceil(6e8 / hv_bytes))))
    hid = [synth.hidden_inputs(cfg.with_(seed=cfg.seed + 1000 * r), "literal", device=dev)
           for r in range(n_hv)]
    l_v = torch.from_numpy(hid[0]["l_v"]).to(dev)
    w = synth.lm_head(cfg, device=dev)
    draft = torch.from_numpy(synth.draft_ids_uniform(cfg)).to(dev)

    # a draft tree stores the rows of its chains one after the other: attention and relevance see
    # gamma rows per sequence, the accept call sees B * n_branches chains of chain_len rows
    n_br, K = cfg.n_branches, cfg.chain_len
    chains = cfg.B * n_br
    tree_mask = cfg.tree_mask()
    draft = draft.reshape(chains, K)
    out = torch.empty((cfg.B, cfg.gamma, cfg.Hq, cfg.D), dtype=torch.bfloat16, device=dev)
    rel = torch.empty((cfg.B, cfg.gamma), dtype=torch.float32, device=dev)
    acc_outs = L.alloc_accept_outputs(chains, K, cfg.V, 4, dev, n_branches=n_br)

    attn_args = []
    for s in kv_sets:
        a = L.verify_attn_args(s["q"], s["k"], s["v"], kv_len, out=out, vis_begin=vis_b,
                               vis_end=vis_e, max_kv_len=max(cfg.kv_len),
                               kv_len_host=list(cfg.kv_len), draft_mask=tree_mask)
        attn_args.append(a)
    ws_attn = torch.empty((max(256, lib.lvspec_verify_attn_workspace(C.byref(attn_args[0]))),),
                          dtype=torch.uint8, device=dev)
    for a in attn_args:
        a.workspace, a.workspace_bytes = ws_attn.data_ptr(), ws_attn.numel()
    rel_args = []
    for h in hid:
        a = L.visual_relevance_args(h["h_d"], h["h_v"], l_v, cfg.top_n, relevance=rel)
        rel_args.append(a)
    ws_rel = torch.empty((max(256, lib.lvspec_visual_relevance_workspace(C.byref(rel_args[0]))),),
                         dtype=torch.uint8, device=dev)
    for a in rel_args:
        a.workspace, a.workspace_bytes = ws_rel.data_ptr(), ws_rel.numel()
    acc_args = L.loose_accept_args(hid[0]["h_d"].reshape(chains, K, cfg.d), w, draft,
                                   rel.reshape(chains, K), cfg.n_loose, cfg.pst_window, topk=4,
                                   loose_topk_gate=0, outs=acc_outs, n_branches=n_br)
    ws_acc = torch.empty((max(256, lib.lvspec_loose_accept_workspace(C.byref(acc_args))),),
                         dtype=torch.uint8, device=dev)
    acc_args.workspace, acc_args.workspace_bytes = ws_acc.data_ptr(), ws_acc.numel()

    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    layers = cfg.layers

    def check(rc):
        if rc != 0:
            raise L.LvspecError(rc)

    def run_step(step, events=None):
        if events:
            events[0].record(stream)
        if layers > 1:
            for l in range(layers):
                check(lib.lvspec_verify_attn(C.byref(attn_args[l]), sp))
        else:
            check(lib.lvspec_verify_attn(C.byref(attn_args[step % n_kv]), sp))
        if events:
            events[1].record(stream)
        check(lib.lvspec_visual_relevance(C.byref(rel_args[step % n_hv]), sp))
        if events:
            events[2].record(stream)
        check(lib.lvspec_loose_accept(C.byref(acc_args), sp))
        if events:
            events[3].record(stream)

    if args.calibrate_copy:
        src = torch.zeros((1 << 28,), dtype=torch.int32, device=dev)       # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)          # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for s in range(args.warmup):
        run_step(s)
    torch.cuda.synchronize()

    # ------------------------------------------------------------------ timed region
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_step(s, evs[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / args.steps
    attn_us = np.array([e[0].elapsed_time(e[1]) for e in evs]) * 1e3 / layers
    rel_us = np.array([e[1].elapsed_time(e[2]) for e in evs]) * 1e3
    acc_us = np.array([e[2].elapsed_time(e[3]) for e in evs]) * 1e3
    gpu_ms = float(np.mean([e[0].elapsed_time(e[3]) for e in evs]))
    ms_per_step = wall_ms
    tokens = cfg.B * cfg.gamma

    # ------------------------------------------------------------------ optional graph replay
    graph_ms = None
    if args.graph:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            sp_side = side.cuda_stream
            with torch.cuda.graph(g, stream=side):
                for l in range(layers):
                    check(lib.lvspec_verify_attn(C.byref(attn_args[l % n_kv]), sp_side))
                check(lib.lvspec_visual_relevance(C.byref(rel_args[0]), sp_side))
                check(lib.lvspec_loose_accept(C.byref(acc_args), sp_side))
        torch.cuda.synchronize()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # ------------------------------------------------------------------ rooflines
    # algorithmic bytes: every K/V row once, Q and O once (per layer); H_V + H_D once; W + H_D once
    attn_bytes = layer_bytes + 2 * cfg.B * cfg.gamma * cfg.Hq * cfg.D * 2
    rel_bytes = hv_bytes + cfg.B * cfg.gamma * cfg.d * 2
    lmh_bytes = cfg.V * cfg.d * 2 + cfg.B * cfg.gamma * cfg.d * 2
    traffic = {}
    if os.path.exists(args.traffic_json):
        try:
            traffic = json.load(open(args.traffic_json)).get(cfg.name, {})
        except Exception:
            traffic = {}

    mfma = {}
    if os.path.exists(args.traffic_json):
        try:
            mfma = json.load(open(args.traffic_json)).get(cfg.name + ":mfma", {})
        except Exception:
            mfma = {}

    def roof(nbytes, us, key):
        gbs = nbytes / (us * 1e-6) / 1e9
        # mfma_frac_of_peak: executed bf16 MFMA flops of the streaming kernel over its duration,
        # as a fraction of the 2.5 PFLOP/s dense peak (rocprofv3 counters, see profiles/)
        return {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get(key),
                "algorithmic_bytes": int(nbytes), "avg_us": round(float(us), 2),
                "mfma_frac_of_peak": mfma.get(key, {}).get("frac_of_bf16_peak")}

    roofs = {
        "verify_attn": roof(attn_bytes, float(attn_us.mean()), "verify_attn"),
        "visual_relevance": roof(rel_bytes, float(rel_us.mean()), "visual_relevance"),
        "lm_head_accept": roof(lmh_bytes, float(acc_us.mean()), "lm_head_accept"),
    }
    tot = {"verify_attn": float(attn_us.mean()) * layers, "visual_relevance": float(rel_us.mean()),
           "lm_head_accept": float(acc_us.mean())}
    dominant = max(tot, key=tot.get)

    # ------------------------------------------------------------------ CPU oracle beside it
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_lay = min(layers, 2)
        t_attn = 0.0
        for l in range(n_lay):
            s = kv_sets[l]
            qh, kh, vh = (synth.from_torch_bf16(s[x]) for x in ("q", "k", "v"))
            t = time.perf_counter()
            oracle.verify_attn(qh, kh, vh, s["kv_len"], s["vis_begin"], s["vis_end"],
                               draft_mask=tree_mask)
            t_attn += time.perf_counter() - t
        hd_h, hv_h = synth.from_torch_bf16(hid[0]["h_d"]), synth.from_torch_bf16(hid[0]["h_v"])
        # bound the sample: at most ~6e9 multiply-adds of relevance and of lm_head
        lv_s = int(min(cfg.vis_len, max(1, 6e9 // (cfg.B * cfg.gamma * cfg.d))))
        t = time.perf_counter()
        rel_o = oracle.visual_relevance(hd_h, hv_h[:, :lv_s], np.full(cfg.B, lv_s), cfg.top_n)
        t_rel = (time.perf_counter() - t) * (cfg.vis_len / lv_s)
        v_s = int(min(cfg.V, max(1, 6e9 // (cfg.B * cfg.gamma * cfg.d))))
        w_h = synth.from_torch_bf16(w[:v_s])
        t = time.perf_counter()
        oracle.loose_accept(hd_h.reshape(chains, K, cfg.d), w_h, draft.cpu().numpy() % v_s,
                            rel_o.astype(np.float32).reshape(chains, K), cfg.n_loose,
                            cfg.pst_window, topk=4, n_branches=n_br)
        t_acc = (time.perf_counter() - t) * (cfg.V / v_s)
        step_s = t_attn / n_lay * layers + t_rel + t_acc
        cpu = {"value": round(tokens / step_s, 3), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": (f"{n_lay} of {layers} attention layers, {lv_s} of {cfg.vis_len} video "
                          f"rows of relevance, {v_s} of {cfg.V} vocabulary rows of lm_head+accept; "
                          "each part scaled linearly to the full step"),
               "step_seconds_estimated": round(step_s, 3)}

    res = {
        "metric": "draft tokens verified per second (whole verify step: layers x verify attention "
                  "+ visual relevance + lm_head/loose accept)",
        "value": round(tokens / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "verify_step_latency_us": round(ms_per_step * 1e3, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "gamma": cfg.gamma, "Hq": cfg.Hq,
                   "Hkv": cfg.Hkv, "D": cfg.D, "kv_len": list(cfg.kv_len), "layers": layers,
                   "visual_tokens": cfg.vis_len, "hidden": cfg.d, "vocab": cfg.V,
                   "top_n": cfg.top_n, "n_loose": cfg.n_loose, "pst_window": cfg.pst_window,
                   "draft_tree_branches": n_br, "chain_len": K,
                   "distinct_kv_caches": n_kv},
        "roofline": dict(roofs[dominant], kernel=KERNELS_OF[dominant]),
        "rooflines": roofs,
        "breakdown_us": {"verify_attn_per_layer": round(float(attn_us.mean()), 2),
                         "verify_attn_per_layer_min": round(float(attn_us.min()), 2),
                         "visual_relevance": round(float(rel_us.mean()), 2),
                         "lm_head_accept": round(float(acc_us.mean()), 2),
                         "gpu_step_ms_events": round(gpu_ms, 4)},
        "graph_replay_ms_per_step": None if graph_ms is None else round(graph_ms, 4),
        "cpu_baseline": cpu,
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
