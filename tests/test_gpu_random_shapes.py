"""GPU parity on seeded random shapes: every entry point against the oracle on small inputs whose
shape parameters (batch, heads, group size, draft rows, lengths, spans, draft-tree masks, hidden
size, vocabulary, top-k, Top-N, bonus row, branches) are drawn at random, so that combinations
nobody wrote down as a case get exercised too."""
import numpy as np
import pytest

import oracle
from paper_2604_05650_amd import synth
import test_gpu_accept as acc_cases
import test_gpu_attention as attn_cases
import test_gpu_relevance as rel_cases

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_attention_shapes(seed):
    rng = np.random.default_rng((810, seed))
    for it in range(12):
        Hkv = int(rng.choice([1, 2, 3, 4, 8]))
        G = int(rng.choice([1, 2, 4, 5, 7, 8]))
        gamma = min(int(rng.integers(1, 33)), 256 // G)
        B = int(rng.integers(1, 4))
        lmax = int(rng.choice([0, 5, 40, 200, 1000, 3000]))
        kv_len = rng.integers(0, lmax + 1, B).astype(np.int32)
        cap = int(kv_len.max()) + gamma + int(rng.integers(0, 5))
        q = synth.normal_bf16((811, seed, it, 0), (B, gamma, Hkv * G, 128), 1.0)
        k = synth.normal_bf16((811, seed, it, 1), (B, Hkv, cap, 128), 1.0)
        v = synth.normal_bf16((811, seed, it, 2), (B, Hkv, cap, 128), 1.0)
        vb = np.array([rng.integers(0, kv_len[b] + 1) for b in range(B)], np.int32)
        ve = np.array([rng.integers(vb[b], kv_len[b] + 1) for b in range(B)], np.int32)
        mask = None
        if gamma >= 2 and rng.random() < 0.5:
            # a random forest over the draft rows: row i sees itself and what its parent sees
            mask = np.zeros(gamma, np.uint32)
            for i in range(gamma):
                parent = int(rng.integers(-1, i))
                mask[i] = (mask[parent] if parent >= 0 else 0) | (1 << i)
        attn_cases._check(q, k, v, kv_len, vb, ve, draft_mask=mask, tag=f"random {seed}.{it}")


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_random_relevance_shapes(seed):
    rng = np.random.default_rng((820, seed))
    for it in range(12):
        B, g = int(rng.integers(1, 4)), int(rng.integers(1, 33))
        d = int(rng.choice([128, 256, 384, 512, 1024, 2048]))
        lv_max = int(rng.choice([1, 17, 64, 300, 1500, 5000, 20000]))
        top_n = int(rng.choice([1, 5, 10, 16, 17, 100]))
        h_d = synth.normal_bf16((821, seed, it, 0), (B, g, d), 1.0)
        h_v = synth.normal_bf16((821, seed, it, 1), (B, lv_max, d), 1.0)
        l_v = rng.integers(0, lv_max + 1, B).tolist()
        l_v[0] = lv_max
        rel_cases._check(h_d, h_v, l_v, top_n, f"random {seed}.{it}")


@pytest.mark.parametrize("seed", [31, 32, 33])
def test_random_accept_shapes(seed):
    rng = np.random.default_rng((830, seed))
    for it in range(12):
        n_br = int(rng.choice([1, 1, 2, 3]))
        bonus = bool(rng.random() < 0.5)
        K = int(rng.integers(1, 17))
        while n_br * (K + bonus) > 48:
            K -= 1
        chains = int(rng.integers(1, 5)) * n_br
        V = int(rng.choice([50, 129, 1000, 5000, 33000]))
        d = int(rng.choice([128, 256, 640, 4096]))
        topk = int(min(V, rng.choice([1, 2, 4, 16])))
        h_d = synth.normal_bf16((831, seed, it, 0), (chains, K + (1 if bonus else 0), d), 1.0)
        w = synth.normal_bf16((831, seed, it, 1), (V, d), 0.05)
        h_d, planted = synth.plant_target_rows(h_d, w, 30.0, (831, seed, it, 2))
        draft = synth.draft_ids_from_target(planted[:, :K], (831, seed, it, 3), p_wrong=0.3, V=V)
        rel = synth.bf16_bits_to_f32(synth.normal_bf16((831, seed, it, 4), (chains, K), 1.0))
        acc_cases._check(h_d, w, draft, rel, oracle.n_loose(0.7, K), int(rng.integers(0, K + 1)),
                         topk=topk, logits=V <= 5000, tag=f"random {seed}.{it}", bonus_row=bonus,
                         n_branches=n_br)
