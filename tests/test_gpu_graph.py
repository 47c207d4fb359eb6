"""The three entry points only enqueue kernels (no allocation, no memset, no host sync), so a
whole verify step can be captured into a HIP graph.  Every replay must reproduce the eager
results bit for bit, also after the inputs were overwritten in place and with eager work and
synchronisations between the replays."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2604_05650_amd import synth
from parity import dev, t_bf16, t_f32, t_i32, to_np

pytestmark = pytest.mark.gpu


def test_captured_step_replays_bit_exact():
    from paper_2604_05650_amd import binding as L
    lib = L.raw()
    cfg = synth.CONFIGS["c1"]
    a = synth.attn_inputs(cfg)
    h = synth.hidden_inputs(cfg, "structured")
    w = t_bf16(synth.lm_head(cfg))
    q, k, v = t_bf16(a["q"]), t_bf16(a["k"]), t_bf16(a["v"])
    kv_len, vb, ve = t_i32(a["kv_len"]), t_i32(a["vis_begin"]), t_i32(a["vis_end"])
    h_d, h_v, l_v = t_bf16(h["h_d"]), t_bf16(h["h_v"]), t_i32(h["l_v"])
    draft = t_i32(synth.draft_ids_uniform(cfg))
    out = torch.empty_like(q)
    lse = torch.empty((cfg.B, cfg.Hq, cfg.gamma), dtype=torch.float32, device=dev())
    rel = torch.empty((cfg.B, cfg.gamma), dtype=torch.float32, device=dev())
    outs = L.alloc_accept_outputs(cfg.B, cfg.gamma, cfg.V, 4, dev())

    aa = L.verify_attn_args(q, k, v, kv_len, out=out, vis_begin=vb, vis_end=ve, lse=lse)
    ra = L.visual_relevance_args(h_d, h_v, l_v, cfg.top_n, relevance=rel)
    ca = L.loose_accept_args(h_d, w, draft, rel, cfg.n_loose, cfg.pst_window, topk=4,
                             loose_topk_gate=0, outs=outs)
    wss = []
    for args, fn in ((aa, lib.lvspec_verify_attn_workspace),
                     (ra, lib.lvspec_visual_relevance_workspace),
                     (ca, lib.lvspec_loose_accept_workspace)):
        ws = torch.empty((max(256, fn(C.byref(args))),), dtype=torch.uint8, device=dev())
        args.workspace, args.workspace_bytes = ws.data_ptr(), ws.numel()
        wss.append(ws)

    def enqueue(stream_ptr):
        for args, fn in ((aa, lib.lvspec_verify_attn), (ra, lib.lvspec_visual_relevance),
                         (ca, lib.lvspec_loose_accept)):
            rc = fn(C.byref(args), stream_ptr)
            assert rc == 0, L.status_string(rc)

    def snapshot():
        torch.cuda.synchronize()
        r = {"out": out.view(torch.int16).cpu().numpy().copy(), "lse": lse.cpu().numpy().copy(),
             "rel": rel.cpu().numpy().copy()}
        r.update({k_: v_.copy() for k_, v_ in to_np(outs).items()})
        return r

    def eager():
        enqueue(torch.cuda.current_stream().cuda_stream)
        return snapshot()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            enqueue(side.cuda_stream)
    torch.cuda.synchronize()

    rng = np.random.default_rng(5)
    for it in range(4):
        if it > 0:   # new inputs in place: the graph holds pointers, not values
            q.copy_(t_bf16(synth.normal_bf16((900, it, 0), tuple(q.shape), cfg.qkv_std)))
            h_d.copy_(t_bf16(synth.normal_bf16((900, it, 1), tuple(h_d.shape), 1.0)))
            draft.copy_(t_i32(rng.integers(0, cfg.V, (cfg.B, cfg.gamma))))
        want = eager()
        for t in (out, lse, rel):          # scribble over the outputs between eager and replay
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for key in want:
            np.testing.assert_array_equal(got[key], want[key], err_msg=f"replay {it}: {key}")
    # and the last replay agrees with the oracle (attention rows)
    o_out, _, _ = oracle.verify_attn(synth.from_torch_bf16(q), a["k"], a["v"], a["kv_len"])
    g_out = out.float().cpu().numpy().astype(np.float64)
    err = np.abs(g_out - o_out).max(-1) / np.abs(o_out).max(-1)
    assert err.max() <= 1e-2
