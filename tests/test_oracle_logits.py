"""Pins for oracle O3 (lm_head logits, greedy token, softmax statistics, top-k)."""
import numpy as np
import torch

import oracle
from paper_2604_05650_amd import synth


def test_logits_match_library_matmul():
    rows, d, V = 5, 48, 301
    h = synth.normal_bf16((1, 0), (rows, d), 1.0)
    w = synth.normal_bf16((1, 1), (V, d), 0.02)
    z = oracle.logits(h, w)
    ref = (torch.from_numpy(synth.bf16_bits_to_f32(h)).double()
           @ torch.from_numpy(synth.bf16_bits_to_f32(w)).double().T).numpy()
    np.testing.assert_allclose(z, ref, rtol=1e-12, atol=1e-15)
    cols = [0, 7, 300, 123]
    np.testing.assert_array_equal(oracle.logits(h, w, cols=cols), z[:, cols])


def test_unit_vectors_pick_matrix_entries():
    # h = e_t  =>  z_v = W[v, t]: catches a transposed operand or wrong stride
    d, V = 8, 11
    w = synth.normal_bf16((2, 1), (V, d), 1.0)
    h = synth.f32_to_bf16_bits(np.eye(d, dtype=np.float32))
    z = oracle.logits(h, w)
    np.testing.assert_array_equal(z, synth.bf16_bits_to_f32(w).astype(np.float64).T)


def test_planted_row_wins_argmax():
    d, V = 64, 500
    w = synth.normal_bf16((3, 1), (V, d), 0.02)
    w64 = synth.bf16_bits_to_f32(w).astype(np.float64)
    gram = w64 @ w64.T
    for vstar in (0, 17, 499):
        assert np.all(np.delete(gram[vstar], vstar) < gram[vstar, vstar])
        h = synth.f32_to_bf16_bits((4.0 * synth.bf16_bits_to_f32(w[vstar]))[None])
        r = oracle.softmax_topk(oracle.logits(h, w)[0], 3)
        assert r["y"] == vstar and r["topk_ids"][0] == vstar


def test_softmax_statistics_and_topk():
    rng = np.random.default_rng(7)
    z = rng.normal(size=777) * 3
    r = oracle.softmax_topk(z, 16)
    p = torch.softmax(torch.from_numpy(z), 0)
    tv, ti = torch.topk(p, 16)
    np.testing.assert_array_equal(r["topk_ids"], ti.numpy())
    np.testing.assert_allclose(r["topk_probs"], tv.numpy(), rtol=1e-12)
    assert abs(r["lse"] - torch.logsumexp(torch.from_numpy(z), 0).item()) < 1e-12
    assert abs(r["entropy"] - float(-(p * p.log()).sum())) < 1e-12
    zs = np.sort(z)
    assert abs(r["margin"] - (zs[-1] - zs[-2]) / np.abs(z).max()) < 1e-15
    # all probabilities (k = V) sum to one
    full = oracle.softmax_topk(z[:50], 50)
    assert abs(full["topk_probs"].sum() - 1.0) < 1e-12
    # uniform logits: entropy ln V, lowest id first
    u = oracle.softmax_topk(np.full(64, 2.5), 4)
    assert abs(u["entropy"] - np.log(64)) < 1e-12 and abs(u["lse"] - (2.5 + np.log(64))) < 1e-12
    np.testing.assert_array_equal(u["topk_ids"], [0, 1, 2, 3])


def test_ties_go_to_lowest_id_in_binary32():
    z = np.zeros(10)
    z[[3, 6]] = 1.0
    z[6] += 1e-12            # equal once rounded to binary32, the precision of the decision
    r = oracle.softmax_topk(z, 2)
    assert r["y"] == 3 and list(r["topk_ids"]) == [3, 6]


def test_loose_accept_chain_on_tiny_case():
    # compose O3 -> O4 -> O5 by hand on a 3-token vocabulary and compare with the chain
    d, V = 4, 3
    w = synth.f32_to_bf16_bits(np.array([[1, 0, 0, 0], [0, 1, 0, 0], [0, 0, 1, 0]], np.float32))
    h = synth.f32_to_bf16_bits(np.array([[[2, 1, 0, 0], [0, 3, 1, 0], [1, 0, 2, 0]]], np.float32))
    # targets: 0, 1, 2 ; drafts 0, 2, 1 ; relevance lowest at position 1
    out = oracle.loose_accept(h, w, [[0, 2, 1]], [[0.9, 0.1, 0.5]], n_loose_=1, pst_window=0,
                              topk=2)
    np.testing.assert_array_equal(out["target_ids"], [[0, 1, 2]])
    np.testing.assert_array_equal(out["verdict"], [[1, 2, 0]])
    assert out["accept_len"][0] == 2 and out["bonus_id"][0] == 2
    np.testing.assert_array_equal(out["topk_ids"][0, 1], [1, 2])
    out = oracle.loose_accept(h, w, [[0, 2, 1]], [[0.9, 0.1, 0.5]], n_loose_=1, pst_window=1,
                              topk=2)
    np.testing.assert_array_equal(out["verdict"], [[1, 2, 3]])
    assert out["accept_len"][0] == 3 and out["bonus_id"][0] == -1
    assert abs(out["loose_margin"][0] - (0.5 - 0.1) / 0.9) < 1e-6
    # gate: loosened position 1 drafted token 2 is the row's 2nd choice -> inside top-2, not top-1
    out = oracle.loose_accept(h, w, [[0, 2, 1]], [[0.9, 0.1, 0.5]], 1, 0, topk=2,
                              loose_topk_gate=1)
    np.testing.assert_array_equal(out["verdict"], [[1, 0, 0]])
    out = oracle.loose_accept(h, w, [[0, 2, 1]], [[0.9, 0.1, 0.5]], 1, 0, topk=2,
                              loose_topk_gate=2)
    np.testing.assert_array_equal(out["verdict"], [[1, 2, 0]])


def test_entropy_closed_forms():
    # two tokens with odds 1:3 -> H = -(1/4 ln 1/4 + 3/4 ln 3/4); a one-hot row -> 0;
    # adding a constant to every logit changes nothing
    r = oracle.softmax_topk(np.array([0.0, np.log(3.0)]), 2)
    h = -(0.25 * np.log(0.25) + 0.75 * np.log(0.75))
    assert abs(r["entropy"] - h) < 1e-12
    assert abs(oracle.softmax_topk(np.array([0.0, np.log(3.0)]) + 123.0, 2)["entropy"] - h) < 1e-9
    assert oracle.softmax_topk(np.array([800.0, 0.0, 0.0]), 1)["entropy"] < 1e-300
    v = 1000
    assert abs(oracle.softmax_topk(np.zeros(v), 1)["entropy"] - np.log(v)) < 1e-12
