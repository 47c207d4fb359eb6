"""GPU integration: several verify steps in a row, the state carried on the device.

Each step appends the draft rows' K/V behind the cache, runs verification attention (one layer),
the relevance of the drafts' hidden rows (rows 1..gamma of the step's gamma+1 final rows), the
loose acceptance with the bonus row (rows 0..gamma), and commits the kept chain to the cache; the
next step starts from the committed lengths.  The "models" are synthetic (seeded rows per step),
so the chain exercises the plumbing between the four entry points, not a transformer.  The same
chain runs through the oracle (O1, O2, O3-O6, O7) step by step; decisions are compared bit for
bit (targets are planted with wide margins), attention outputs within the float tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_05650_amd import synth
from parity import TOL, assert_rows_close, assert_scalars_close, t_bf16, t_f32, t_i32

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_br,K", [(1, 4), (2, 3)])
def test_decode_loop(n_br, K):
    from paper_2604_05650_amd import binding as L
    B, Hq, Hkv, D, d, V, lv, steps = 2, 8, 2, 128, 256, 3000, 700, 5
    gamma = n_br * K
    cap = 900 + steps * gamma
    n_loose = oracle.n_loose(0.7, K)
    mask = synth.branch_mask(n_br, K) if n_br > 1 else None
    # device state
    k_o = synth.normal_bf16((701, n_br, 0), (B, Hkv, cap, D), 0.5)
    v_o = synth.normal_bf16((701, n_br, 1), (B, Hkv, cap, D), 0.5)
    len_o = np.array([800, 333], np.int32)
    k_g, v_g, len_g = t_bf16(k_o), t_bf16(v_o), t_i32(len_o)
    next_len = torch.empty_like(len_g)
    h_v = synth.normal_bf16((701, n_br, 2), (B, lv, d), 1.0)
    w = synth.normal_bf16((701, n_br, 3), (V, d), 0.05)
    l_v = np.array([lv, lv - 100], np.int32)
    h_v_g, w_g, l_v_g = t_bf16(h_v), t_bf16(w), t_i32(l_v)
    vis_b, vis_e = np.array([8, 8], np.int32), np.array([8 + lv, lv - 92], np.int32)
    total_accepted = 0
    compared = 0
    for s in range(steps):
        print(f"[loop] br{n_br} K{K} step {s} lens {len_o.tolist()}", flush=True)
        # the step's synthetic model outputs: draft K/V rows, queries, final hidden rows
        q = synth.normal_bf16((702, s, 0), (B, gamma, Hq, D), 0.5)
        dk = synth.normal_bf16((702, s, 1), (B, Hkv, gamma, D), 0.5)
        dv = synth.normal_bf16((702, s, 2), (B, Hkv, gamma, D), 0.5)
        rows = synth.normal_bf16((702, s, 3), (B * n_br, K + 1, d), 1.0)
        # distinct relevance scores: every draft row leans on one video row by its own amount
        rng = np.random.default_rng((703, s, n_br))
        r32 = synth.bf16_bits_to_f32(rows)
        beta = rng.permutation(np.linspace(0.3, 2.4, B * n_br * K)).reshape(B * n_br, K)
        pick = rng.integers(0, lv - 100, (B * n_br, K))
        hv32 = synth.bf16_bits_to_f32(h_v)
        for c in range(B * n_br):
            r32[c, 1:] += beta[c][:, None].astype(np.float32) * hv32[c // n_br, pick[c]]
        rows = synth.f32_to_bf16_bits(r32)
        rows, planted = synth.plant_target_rows(rows, w, 30.0, (702, s, 4))
        draft = synth.draft_ids_from_target(planted[:, :K], (702, s, 5), p_wrong=0.35, V=V)
        if s == 1:
            draft[:] = planted[:, :K]          # a step in which every draft is accepted
        for b in range(B):
            k_o[b, :, len_o[b]:len_o[b] + gamma] = dk[b]
            v_o[b, :, len_o[b]:len_o[b] + gamma] = dv[b]
        # the GPU writes the draft rows at its own (device-side) lengths
        lens_now = len_g.cpu().numpy()
        np.testing.assert_array_equal(lens_now, len_o)
        for b in range(B):
            k_g[b, :, lens_now[b]:lens_now[b] + gamma] = t_bf16(dk[b])
            v_g[b, :, lens_now[b]:lens_now[b] + gamma] = t_bf16(dv[b])
        # ---- GPU step
        out_g = L.verify_attn(t_bf16(q), k_g, v_g, len_g, vis_begin=t_i32(vis_b),
                              vis_end=t_i32(vis_e), draft_mask=mask)
        rows_g = t_bf16(rows).view(B * n_br, K + 1, d)
        rel_in = rows_g[:, 1:].reshape(B, gamma, d).contiguous() if n_br > 1 else rows_g[:, 1:]
        rel_g = L.visual_relevance(rel_in, h_v_g, l_v_g, 10)
        res = L.loose_accept(rows_g, w_g, t_i32(draft), rel_g.view(B * n_br, K), n_loose, K,
                             topk=2, n_branches=n_br, bonus_row=True)
        L.kv_commit(k_g, v_g, len_g, res["accept_len"], K, best_branch=res.get("best_branch"),
                    n_branches=n_br, new_len=next_len)
        len_g, next_len = next_len, len_g
        torch.cuda.synchronize()
        # ---- oracle step
        out_o, _, _ = oracle.verify_attn(q, k_o, v_o, len_o, vis_b, vis_e, draft_mask=mask)
        rel_o = oracle.visual_relevance(
            np.ascontiguousarray(rows[:, 1:]).reshape(B, gamma, d), h_v, l_v, 10)
        acc_o = oracle.loose_accept(rows, w, draft, rel_o.astype(np.float32).reshape(B * n_br, K),
                                    n_loose, K, topk=2, n_branches=n_br, bonus_row=True)
        assert acc_o["margin"].min() > TOL
        best_o = acc_o.get("best_branch")
        k_o, v_o, len_o = oracle.kv_commit(k_o, v_o, len_o, acc_o["accept_len"], K,
                                           best_branch=best_o, n_branches=n_br)
        # ---- compare
        g_out = out_g.float().cpu().numpy().astype(np.float64)
        assert_rows_close(g_out.reshape(-1, D), out_o.reshape(-1, D), f"attention step {s}")
        assert_scalars_close(rel_g.cpu().numpy(), rel_o, f"relevance step {s}")
        np.testing.assert_array_equal(res["target_ids"].cpu().numpy(), planted)
        if np.all(acc_o["loose_margin"] > TOL):
            compared += 1
            np.testing.assert_array_equal(res["verdict"].cpu().numpy(), acc_o["verdict"])
            np.testing.assert_array_equal(res["accept_len"].cpu().numpy(), acc_o["accept_len"])
            np.testing.assert_array_equal(res["bonus_id"].cpu().numpy(), acc_o["bonus_id"])
            if n_br > 1:
                np.testing.assert_array_equal(res["best_branch"].cpu().numpy(), best_o)
            np.testing.assert_array_equal(len_g.cpu().numpy(), len_o)
        else:   # a relevance near-tie at the loosened-set boundary: follow the oracle's state
            len_g.copy_(t_i32(len_o))
            k_g.copy_(t_bf16(k_o)); v_g.copy_(t_bf16(v_o))
        for b in range(B):
            np.testing.assert_array_equal(
                synth.from_torch_bf16(k_g[b, :, :len_o[b]].contiguous()), k_o[b, :, :len_o[b]])
        total_accepted += int(acc_o["accept_len"].sum())
        if s == 1:
            kept = acc_o["accept_len"].reshape(B, n_br).max(1)
            assert np.all(kept == K) and np.all(acc_o["bonus_id"] >= 0)
    print(f"[loop] br{n_br} K{K}: decisions compared in {compared} of {steps} steps, "
          f"{total_accepted} tokens accepted", flush=True)
    assert total_accepted > 0 and compared >= 2
