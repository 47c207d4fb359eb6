"""GPU parity of the draft-tree step (appendix on draft token trees): tree-masked verification
attention over all chains' rows, relevance of up to 32 draft rows in one pass, per-chain loose
acceptance and the choice of the longest chain, each against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from golden_io import tree_cases
from paper_2604_05650_amd import synth
from parity import (assert_rows_close, assert_scalars_close, bf16_out_to_f64, compare_accept, dev,
                    t_bf16, t_f32, t_i32, to_np)

pytestmark = pytest.mark.gpu


def _attn(q, k, v, kv_len, mask, vb=None, ve=None):
    from paper_2604_05650_amd import binding as L
    out, lse, vm = L.verify_attn(t_bf16(q), t_bf16(k), t_bf16(v), t_i32(kv_len), draft_mask=mask,
                                 vis_begin=None if vb is None else t_i32(vb),
                                 vis_end=None if ve is None else t_i32(ve),
                                 return_lse=True, return_vis_mass=vb is not None)
    torch.cuda.synchronize()
    return bf16_out_to_f64(out), lse.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("Hq,Hkv,n_br,K,L", [(40, 8, 2, 10, 1000), (8, 2, 2, 16, 333),
                                             (4, 4, 3, 7, 95), (64, 8, 2, 10, 31),
                                             (2, 1, 4, 8, 0)])
def test_tree_attention(Hq, Hkv, n_br, K, L):
    B, D, gamma = 1, 128, n_br * K
    cap = L + gamma + 5
    q = synth.normal_bf16((501, Hq, K, L, 0), (B, gamma, Hq, D), 1.0)
    k = synth.normal_bf16((501, Hq, K, L, 1), (B, Hkv, cap, D), 1.0)
    v = synth.normal_bf16((501, Hq, K, L, 2), (B, Hkv, cap, D), 1.0)
    mask = synth.branch_mask(n_br, K)
    print(f"[tree] attn Hq{Hq} Hkv{Hkv} {n_br}x{K} L{L}", flush=True)
    g_out, g_lse = _attn(q, k, v, [L], mask)
    o_out, o_lse, _ = oracle.verify_attn(q, k, v, [L], draft_mask=mask)
    e1 = assert_rows_close(g_out, o_out, "tree attn out")
    e2 = assert_scalars_close(g_lse, o_lse, "tree attn lse")
    print(f"[tree] ok out {e1:.2e} lse {e2:.2e}", flush=True)


@pytest.mark.parametrize("gamma", [17, 24, 32])
def test_chain_attention_beyond_sixteen_rows(gamma):
    B, Hq, Hkv, D, L = 2, 6, 2, 128, 150
    cap = L + gamma
    q = synth.normal_bf16((502, gamma, 0), (B, gamma, Hq, D), 1.0)
    k = synth.normal_bf16((502, gamma, 1), (B, Hkv, cap, D), 1.0)
    v = synth.normal_bf16((502, gamma, 2), (B, Hkv, cap, D), 1.0)
    print(f"[tree] causal rows {gamma}", flush=True)
    g_out, g_lse = _attn(q, k, v, [L, 17], None)
    o_out, o_lse, _ = oracle.verify_attn(q, k, v, [L, 17])
    assert_rows_close(g_out, o_out, "causal >16 rows out")
    assert_scalars_close(g_lse, o_lse, "causal >16 rows lse")


@pytest.mark.parametrize("B,gamma,lv,d", [(2, 17, 130, 256), (2, 20, 1000, 640),
                                          (2, 32, 77, 128), (2, 32, 4100, 1024),
                                          (8, 20, 8200, 128)])
def test_relevance_of_all_tree_rows(B, gamma, lv, d):
    from paper_2604_05650_amd import binding as L
    h_d = synth.normal_bf16((503, gamma, lv, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((503, gamma, lv, 1), (B, lv, d), 1.0)
    l_v = [lv if b % 2 == 0 else max(lv // 3, 1) for b in range(B)]
    print(f"[tree] relevance g{gamma} lv{lv} d{d}", flush=True)
    rel = L.visual_relevance(t_bf16(h_d), t_bf16(h_v), t_i32(l_v), 10)
    torch.cuda.synchronize()
    o = oracle.visual_relevance(h_d, h_v, l_v, 10)
    e = assert_scalars_close(rel.cpu().numpy(), o, "tree relevance")
    print(f"[tree] ok {e:.2e}", flush=True)


def _accept(h_d, w, draft, rel, n_loose, pst, n_br, topk=2):
    from paper_2604_05650_amd import binding as L
    outs = L.loose_accept(t_bf16(h_d), t_bf16(w), t_i32(draft), t_f32(rel), n_loose, pst,
                          topk=topk, n_branches=n_br)
    torch.cuda.synchronize()
    return to_np(outs)


@pytest.mark.parametrize("case", tree_cases(), ids=[c["name"] for c in tree_cases()])
def test_hand_tree_cases_through_the_library(case):
    # target ids planted through near-one-hot hidden rows on a small vocabulary
    d, V = 128, 130
    w32 = np.zeros((V, d), np.float32)
    w32[np.arange(V), np.arange(V) % d] = 1.0
    w32[np.arange(V), (np.arange(V) // d + 7 * np.arange(V) + 1) % d] += 0.5
    w = synth.f32_to_bf16_bits(w32)
    ch = case["chains"]
    y = np.stack([c["y"] for c in ch])
    dr = np.stack([c["d"] for c in ch])
    a = np.stack([c["a"] for c in ch])
    h_d = synth.f32_to_bf16_bits(8.0 * w32[y])
    n_br = len(ch)
    print(f"[tree] {case['name']}", flush=True)
    g = _accept(h_d, w, dr, a, case["n_loose"], case["pst_window"], n_br)
    np.testing.assert_array_equal(g["target_ids"], y)
    np.testing.assert_array_equal(g["accept_len"], case["tau"])
    if n_br > 1:
        assert g["best_branch"].tolist() == [case["kept"]]
    o = oracle.loose_accept(h_d, w, dr, a, case["n_loose"], case["pst_window"], topk=2,
                            n_branches=n_br)
    np.testing.assert_array_equal(g["verdict"], o["verdict"])
    np.testing.assert_array_equal(g["bonus_id"], o["bonus_id"])


@pytest.mark.parametrize("S,n_br,K", [(1, 2, 10), (2, 2, 8), (4, 8, 1), (2, 4, 4), (3, 3, 3)])
def test_random_trees_against_the_oracle(S, n_br, K):
    B, d, V = S * n_br, 256, 3000
    h_d = synth.normal_bf16((504, S, n_br, K, 0), (B, K, d), 1.0)
    w = synth.normal_bf16((504, S, n_br, K, 1), (V, d), 0.05)
    h_d, planted = synth.plant_target_rows(h_d, w, 30.0, (504, S, n_br, K, 2))
    draft = synth.draft_ids_from_target(planted, (504, S, n_br, K, 3), p_wrong=0.25, V=V)
    rel = synth.bf16_bits_to_f32(synth.normal_bf16((504, S, n_br, K, 4), (B, K), 1.0))
    n_loose = oracle.n_loose(0.7, K)
    print(f"[tree] random S{S} {n_br}x{K}", flush=True)
    g = _accept(h_d, w, draft, rel, n_loose, K, n_br, topk=4)
    o = oracle.loose_accept(h_d, w, draft, rel, n_loose, K, topk=4, n_branches=n_br)
    st = compare_accept(g, o, draft, K)
    assert st["counted_sequences"] == B, st
    np.testing.assert_array_equal(g["best_branch"], o["best_branch"])


def test_tree_step_chained_tiny():
    """Whole tree step on the tiny shape: attention with the tree mask, relevance of all rows in
    one call, per-chain acceptance; every stage from the GPU's own previous stage."""
    from paper_2604_05650_amd import binding as L
    cfg = synth.CONFIGS["c1t"]
    a = synth.attn_inputs(cfg)
    mask = cfg.tree_mask()
    g_out, g_lse = _attn(a["q"], a["k"], a["v"], a["kv_len"], mask, a["vis_begin"], a["vis_end"])
    o_out, o_lse, _ = oracle.verify_attn(a["q"], a["k"], a["v"], a["kv_len"], a["vis_begin"],
                                         a["vis_end"], draft_mask=mask)
    assert_rows_close(g_out, o_out, "c1t attn")
    h = synth.hidden_inputs(cfg, "structured")
    w = synth.lm_head(cfg)
    h_d, planted = synth.plant_target_rows(h["h_d"], w, 24.0, (cfg.seed, 77))
    n_br, K = cfg.n_branches, cfg.chain_len
    planted = planted.reshape(n_br, K)
    draft = synth.draft_ids_from_target(planted, (cfg.seed, 78), p_wrong=0.3, V=cfg.V)
    rel = L.visual_relevance(t_bf16(h_d), t_bf16(h["h_v"]), t_i32(h["l_v"]), cfg.top_n)
    o_rel = oracle.visual_relevance(h_d, h["h_v"], h["l_v"], cfg.top_n)
    assert_scalars_close(rel.cpu().numpy(), o_rel, "c1t relevance")
    chains = t_bf16(h_d).reshape(n_br, K, cfg.d)
    outs = to_np(L.loose_accept(chains, t_bf16(w), t_i32(draft), rel.reshape(n_br, K),
                                cfg.n_loose, cfg.pst_window, topk=4, n_branches=n_br))
    o = oracle.loose_accept(h_d.reshape(n_br, K, cfg.d), w, draft,
                            o_rel.astype(np.float32).reshape(n_br, K), cfg.n_loose,
                            cfg.pst_window, topk=4, n_branches=n_br)
    st = compare_accept(outs, o, draft, K)
    assert st["counted_sequences"] == n_br, st
    np.testing.assert_array_equal(outs["best_branch"], o["best_branch"])


def test_tree_full_size_32b_layer():
    """Two chains of ten tokens on the 32B shape, in the launch configuration the benchmark
    times; the oracle computes a seeded sample of the attention rows and the full relevance."""
    from paper_2604_05650_amd import binding as L
    cfg = synth.CONFIGS["c2t"]
    a = synth.attn_inputs(cfg, device=dev())
    mask = cfg.tree_mask()
    print("[tree] c2t launching", flush=True)
    out, lse, _ = L.verify_attn(a["q"], a["k"], a["v"], t_i32(a["kv_len"]), draft_mask=mask,
                                return_lse=True, kv_len_host=a["kv_len"])
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    n = 160
    rows = np.stack([np.zeros(n, np.int64), rng.integers(0, cfg.gamma, n),
                     rng.integers(0, cfg.Hq, n)], 1).astype(np.int32)
    rows[0] = (0, cfg.gamma - 1, cfg.Hq - 1)
    rows[1] = (0, cfg.chain_len, 0)            # first row of the second chain
    rows[2] = (0, cfg.chain_len - 1, 3)        # last row of the first chain
    qh, kh, vh = (synth.from_torch_bf16(a[x]) for x in ("q", "k", "v"))
    o_out, o_lse, _ = oracle.verify_attn(qh, kh, vh, a["kv_len"], draft_mask=mask, rows=rows)
    g = bf16_out_to_f64(out)
    gl = lse.cpu().numpy()
    e1 = assert_rows_close(np.stack([g[b, i, h] for b, i, h in rows]), o_out, "c2t out")
    e2 = assert_scalars_close([gl[b, h, i] for b, i, h in rows], o_lse, "c2t lse")
    h = synth.hidden_inputs(cfg, "structured", device=dev())
    rel = L.visual_relevance(h["h_d"], h["h_v"], t_i32(h["l_v"]), cfg.top_n)
    torch.cuda.synchronize()
    o_rel = oracle.visual_relevance(synth.from_torch_bf16(h["h_d"]),
                                    synth.from_torch_bf16(h["h_v"]), h["l_v"], cfg.top_n)
    e3 = assert_scalars_close(rel.cpu().numpy(), o_rel, "c2t relevance")
    print(f"[tree] c2t ok: out {e1:.2e} lse {e2:.2e} rel {e3:.2e}", flush=True)
