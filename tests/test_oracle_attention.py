"""Pins for oracle O1 (verification attention): library routine, closed forms, invariants."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_05650_amd import synth


def _rand_case(seed, B=2, gamma=3, Hq=4, Hkv=2, D=16, kv_len=(9, 5), std=0.7):
    cap = max(kv_len) + gamma
    q = synth.normal_bf16((seed, 0), (B, gamma, Hq, D), std)
    k = synth.normal_bf16((seed, 1), (B, Hkv, cap, D), std)
    v = synth.normal_bf16((seed, 2), (B, Hkv, cap, D), std)
    return q, k, v, np.asarray(kv_len, np.int32)


def _sdpa_reference(q, k, v, kv_len, draft_mask=None):
    """torch CPU scaled_dot_product_attention in float64 with an explicit boolean mask and
    repeat_interleave for the grouped heads (the library routine O1 reduces to)."""
    B, gamma, Hq, D = q.shape
    Hkv, cap = k.shape[1], k.shape[2]
    G = Hq // Hkv
    qf = torch.from_numpy(synth.bf16_bits_to_f32(q)).double().permute(0, 2, 1, 3)
    kf = torch.from_numpy(synth.bf16_bits_to_f32(k)).double().repeat_interleave(G, dim=1)
    vf = torch.from_numpy(synth.bf16_bits_to_f32(v)).double().repeat_interleave(G, dim=1)
    mask = torch.zeros(B, 1, gamma, cap, dtype=torch.bool)
    for b in range(B):
        L = int(kv_len[b])
        mask[b, 0, :, :L] = True
        for i in range(gamma):
            for j in range(gamma):
                vis = (j <= i) if draft_mask is None else bool((int(draft_mask[i]) >> j) & 1)
                mask[b, 0, i, L + j] = vis
    o = torch.nn.functional.scaled_dot_product_attention(qf, kf, vf, attn_mask=mask)
    return o.permute(0, 2, 1, 3).numpy()


@pytest.mark.parametrize("seed,shape", [
    (1, dict()),
    (2, dict(B=1, gamma=5, Hq=6, Hkv=2, D=32, kv_len=(37,))),
    (3, dict(B=3, gamma=1, Hq=2, Hkv=2, D=8, kv_len=(1, 0, 4))),
])
def test_matches_library_sdpa(seed, shape):
    q, k, v, kv_len = _rand_case(seed, **shape)
    out, lse, vm = oracle.verify_attn(q, k, v, kv_len)
    ref = _sdpa_reference(q, k, v, kv_len)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_forest_masks_match_library_sdpa(seed):
    # arbitrary ancestor masks among the draft rows (draft trees): row i sees itself and whatever
    # its parent sees; the library routine gets the same visibility as an explicit mask
    rng = np.random.default_rng((41, seed))
    gamma = int(rng.integers(2, 13))
    mask = np.zeros(gamma, np.uint32)
    for i in range(gamma):
        parent = int(rng.integers(-1, i))
        mask[i] = (mask[parent] if parent >= 0 else 0) | (1 << i)
    q, k, v, kv_len = _rand_case(100 + seed, B=2, gamma=gamma, Hq=6, Hkv=3, D=16, kv_len=(21, 4))
    out, _, _ = oracle.verify_attn(q, k, v, kv_len, draft_mask=mask)
    ref = _sdpa_reference(q, k, v, kv_len, draft_mask=mask)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)


def test_gqa_head_mapping_is_integer_division():
    # with Hkv distinct V tensors that are constant per kv head, output reveals the kv head used
    B, gamma, Hq, Hkv, D, L = 1, 2, 6, 3, 8, 4
    q, k, _, kv_len = _rand_case(5, B, gamma, Hq, Hkv, D, (L,))
    v32 = np.zeros((B, Hkv, L + gamma, D), np.float32)
    for kvh in range(Hkv):
        v32[:, kvh] = kvh + 1
    out, _, _ = oracle.verify_attn(q, k, synth.f32_to_bf16_bits(v32), kv_len)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, :, h, :], h // (Hq // Hkv) + 1, rtol=1e-12)


def test_equal_keys_give_mean_of_visible_values_and_closed_form_lse():
    B, gamma, Hq, Hkv, D, L = 1, 3, 2, 1, 16, 7
    q, _, v, kv_len = _rand_case(7, B, gamma, Hq, Hkv, D, (L,))
    krow = synth.normal_bf16((7, 9), (D,), 0.5)
    k = np.broadcast_to(krow, (B, Hkv, L + gamma, D)).copy()
    out, lse, vm = oracle.verify_attn(q, k, v, kv_len, vis_begin=[0], vis_end=[L + gamma])
    v64 = synth.bf16_bits_to_f32(v).astype(np.float64)
    q64 = synth.bf16_bits_to_f32(q).astype(np.float64)
    k64 = synth.bf16_bits_to_f32(krow).astype(np.float64)
    for i in range(gamma):
        n_vis = L + i + 1
        np.testing.assert_allclose(out[0, i, 0], v64[0, 0, :n_vis].mean(axis=0), rtol=1e-12,
                                   atol=1e-14)
        for h in range(Hq):
            s = (q64[0, i, h] @ k64) / np.sqrt(D)
            assert abs(lse[0, h, i] - (s + np.log(n_vis))) < 1e-12
    # span covering every visible key: the probabilities sum to one
    np.testing.assert_allclose(vm, 1.0, rtol=0, atol=1e-12)


def test_dominant_key_selects_its_value_row():
    B, gamma, Hq, Hkv, D, L = 1, 1, 1, 1, 16, 12
    q32 = np.zeros((B, gamma, Hq, D), np.float32)
    q32[..., 0] = 8.0
    k32 = np.zeros((B, Hkv, L + gamma, D), np.float32)
    k32[0, 0, 5, 0] = 25.0          # score 8*25/4 = 50 against 0 elsewhere
    v = synth.normal_bf16((11, 2), (B, Hkv, L + gamma, D), 1.0)
    out, lse, vm = oracle.verify_attn(synth.f32_to_bf16_bits(q32), synth.f32_to_bf16_bits(k32),
                                      v, [L], vis_begin=[5], vis_end=[6])
    # the other 12 keys carry exp(-50) ~ 2e-22 each
    np.testing.assert_allclose(out[0, 0, 0], synth.bf16_bits_to_f32(v)[0, 0, 5], rtol=0,
                               atol=1e-19)
    assert abs(vm[0, 0, 0] - 1.0) < 1e-15
    assert abs(lse[0, 0, 0] - 50.0) < 1e-12


def test_causality_among_draft_rows():
    q, k, v, kv_len = _rand_case(13, B=1, gamma=4, Hq=2, Hkv=1, D=16, kv_len=(6,))
    base, lse0, _ = oracle.verify_attn(q, k, v, kv_len)
    L = int(kv_len[0])
    for i in range(3):
        k2, v2 = k.copy(), v.copy()
        k2[0, :, L + i + 1:] ^= 0x1234     # scramble later draft rows and the unused tail
        v2[0, :, L + i + 1:] ^= 0x0456
        out, lse, _ = oracle.verify_attn(q, k2, v2, kv_len)
        np.testing.assert_array_equal(out[0, : i + 1], base[0, : i + 1])
        np.testing.assert_array_equal(lse[0, :, : i + 1], lse0[0, :, : i + 1])
        assert not np.array_equal(out[0, i + 1:], base[0, i + 1:])


def test_visual_mass_range_and_empty_span():
    q, k, v, kv_len = _rand_case(17)
    _, _, vm = oracle.verify_attn(q, k, v, kv_len, vis_begin=[2, 1], vis_end=[6, 3])
    assert np.all(vm > 0) and np.all(vm < 1)
    _, _, vm0 = oracle.verify_attn(q, k, v, kv_len, vis_begin=[3, 3], vis_end=[3, 3])
    np.testing.assert_array_equal(vm0, 0.0)
    # complementary spans add up to one
    _, _, va = oracle.verify_attn(q, k, v, kv_len, vis_begin=[0, 0], vis_end=[4, 2])
    _, _, vb = oracle.verify_attn(q, k, v, kv_len, vis_begin=[4, 2], vis_end=[99, 99])
    np.testing.assert_allclose(va + vb, 1.0, atol=1e-12)


def test_lower_triangular_mask_equals_causal_and_tree_equals_separate_chains():
    q, k, v, kv_len = _rand_case(19, B=1, gamma=4, Hq=2, Hkv=1, D=16, kv_len=(5,))
    base = oracle.verify_attn(q, k, v, kv_len)
    tri = [(1 << (i + 1)) - 1 for i in range(4)]
    got = oracle.verify_attn(q, k, v, kv_len, draft_mask=tri)
    for a, b in zip(base, got):
        np.testing.assert_array_equal(a, b)
    ref = _sdpa_reference(q, k, v, kv_len, draft_mask=tri)
    np.testing.assert_allclose(got[0], ref, rtol=1e-12, atol=1e-13)
    # two branches of two tokens sharing the prefix: rows (0,1) and rows (2,3); each branch must
    # equal the chain result obtained with only that branch appended
    tree = [0b0001, 0b0011, 0b0100, 0b1100]
    out_t, lse_t, _ = oracle.verify_attn(q, k, v, kv_len, draft_mask=tree)
    L = 5
    a = oracle.verify_attn(q[:, :2], k[:, :, : L + 2], v[:, :, : L + 2], kv_len)
    np.testing.assert_allclose(out_t[:, :2], a[0], rtol=1e-13, atol=1e-15)
    k_b = np.concatenate([k[:, :, :L], k[:, :, L + 2: L + 4]], axis=2)
    v_b = np.concatenate([v[:, :, :L], v[:, :, L + 2: L + 4]], axis=2)
    b = oracle.verify_attn(q[:, 2:], k_b, v_b, kv_len)
    np.testing.assert_allclose(out_t[:, 2:], b[0], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(lse_t[:, :, 2:], b[1], rtol=1e-13)


def test_row_subset_equals_full():
    q, k, v, kv_len = _rand_case(23)
    out, lse, vm = oracle.verify_attn(q, k, v, kv_len, vis_begin=[1, 0], vis_end=[4, 2])
    rows = [(0, 0, 0), (1, 2, 3), (0, 1, 2)]
    o2, l2, v2 = oracle.verify_attn(q, k, v, kv_len, vis_begin=[1, 0], vis_end=[4, 2], rows=rows)
    for n, (b, i, h) in enumerate(rows):
        np.testing.assert_array_equal(o2[n], out[b, i, h])
        assert l2[n] == lse[b, h, i] and v2[n] == vm[b, h, i]


def test_scale_argument():
    q, k, v, kv_len = _rand_case(29, B=1, gamma=2, Hq=2, Hkv=1, D=16, kv_len=(6,))
    # scale 0: every visible key weighs the same
    out, lse, _ = oracle.verify_attn(q, k, v, kv_len, scale=0.0)
    v64 = synth.bf16_bits_to_f32(v).astype(np.float64)
    np.testing.assert_allclose(out[0, 1, 0], v64[0, 0, :8].mean(axis=0), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse[0, :, 1], np.log(8.0), rtol=1e-13)
