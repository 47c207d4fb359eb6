"""Pins for oracle O2 (visual relevance, Eq. 8)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_05650_amd import synth


def _bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, np.float32))


def test_hand_case_from_the_definition():
    # hd=(1,0); hv = (1,0),(0,1),(1,1),(-1,0): cosines 1, 0, 1/sqrt2, -1 (all values exact in
    # bf16); Top-N means follow by hand
    hd = _bits([[[1.0, 0.0]]])
    hv = _bits([[[1.0, 0.0], [0.0, 1.0], [1.0, 1.0], [-1.0, 0.0]]])
    rel, cos = oracle.visual_relevance(hd, hv, [4], 1, return_cos=True)
    np.testing.assert_allclose(cos[0, 0], [1.0, 0.0, np.sqrt(0.5), -1.0], atol=1e-15)
    assert abs(rel[0, 0] - 1.0) < 1e-15
    assert abs(oracle.visual_relevance(hd, hv, [4], 2)[0, 0] - 0.8535533905932737) < 1e-15
    assert abs(oracle.visual_relevance(hd, hv, [4], 3)[0, 0] - (1 + np.sqrt(0.5)) / 3) < 1e-15
    assert abs(oracle.visual_relevance(hd, hv, [4], 4)[0, 0] - 0.1767766952966369) < 1e-15
    # N beyond l_v uses all l_v rows; l_v = 0 gives 0
    assert abs(oracle.visual_relevance(hd, hv, [4], 50)[0, 0] - 0.1767766952966369) < 1e-15
    assert oracle.visual_relevance(hd, hv, [0], 3)[0, 0] == 0.0
    # only the first l_v rows count
    assert abs(oracle.visual_relevance(hd, hv, [2], 2)[0, 0] - 0.5) < 1e-15


@pytest.mark.parametrize("seed,B,gamma,lv,d,N", [(1, 2, 3, 40, 24, 10), (2, 1, 5, 17, 64, 1),
                                                  (3, 1, 2, 33, 8, 33)])
def test_matches_library_cosine_topk(seed, B, gamma, lv, d, N):
    hd = synth.normal_bf16((seed, 0), (B, gamma, d), 1.0)
    hv = synth.normal_bf16((seed, 1), (B, lv, d), 1.0)
    rel, cos = oracle.visual_relevance(hd, hv, [lv] * B, N, return_cos=True)
    a = torch.from_numpy(synth.bf16_bits_to_f32(hd)).double()
    b = torch.from_numpy(synth.bf16_bits_to_f32(hv)).double()
    c = torch.nn.functional.cosine_similarity(a[:, :, None, :], b[:, None, :, :], dim=-1)
    np.testing.assert_allclose(cos, c.numpy(), rtol=1e-12, atol=1e-14)
    ref = torch.topk(c, N, dim=-1).values.mean(-1).numpy()
    np.testing.assert_allclose(rel, ref, rtol=1e-12, atol=1e-14)


def test_invariants_range_scale_permutation_extremes():
    seed, B, gamma, lv, d = 5, 1, 4, 50, 32
    hd = synth.normal_bf16((seed, 0), (B, gamma, d), 1.0)
    hv = synth.normal_bf16((seed, 1), (B, lv, d), 1.0)
    rel, cos = oracle.visual_relevance(hd, hv, [lv], 10, return_cos=True)
    assert np.all(np.abs(cos) <= 1 + 1e-12) and np.all(np.abs(rel) <= 1 + 1e-12)
    # scaling a row by a power of two is exact in bf16 and must not change its cosine
    hd2 = _bits(synth.bf16_bits_to_f32(hd) * 4.0)
    hv2 = _bits(synth.bf16_bits_to_f32(hv) * 0.125)
    np.testing.assert_allclose(oracle.visual_relevance(hd2, hv2, [lv], 10), rel, rtol=1e-12)
    # permuting the visual rows changes nothing
    perm = np.random.default_rng(0).permutation(lv)
    np.testing.assert_allclose(oracle.visual_relevance(hd, hv[:, perm], [lv], 10), rel,
                               rtol=1e-13)
    # N = 1 is the maximum cosine, N = l_v the plain mean
    np.testing.assert_allclose(oracle.visual_relevance(hd, hv, [lv], 1)[0], cos[0].max(-1),
                               rtol=1e-15)
    np.testing.assert_allclose(oracle.visual_relevance(hd, hv, [lv], lv)[0], cos[0].mean(-1),
                               rtol=1e-12, atol=1e-15)
    # monotone: the mean of the N largest cannot grow with N
    prev = np.inf
    for N in (1, 2, 5, 10, 25, 50):
        cur = oracle.visual_relevance(hd, hv, [lv], N)[0, 0]
        assert cur <= prev + 1e-15
        prev = cur


def test_identical_row_has_cosine_one_and_duplicates_count():
    d = 16
    row = synth.normal_bf16((9, 0), (d,), 1.0)
    other = synth.normal_bf16((9, 1), (3, d), 1.0)
    hv = np.concatenate([row[None], row[None], other], 0)[None]
    rel = oracle.visual_relevance(row[None, None], hv, [5], 2)
    assert abs(rel[0, 0] - 1.0) < 1e-14


def test_zero_rows_use_the_norm_floor():
    hd = _bits(np.zeros((1, 1, 4)))
    hv = _bits([[[1.0, 2.0, 3.0, 4.0], [0.0, 0.0, 0.0, 0.0]]])
    rel = oracle.visual_relevance(hd, hv, [2], 2)
    assert rel[0, 0] == 0.0


# ---- prefill-side inverse norms (O2p) and Eq. 8 with them given -------------------------------
def test_inverse_norms_hand_case_and_floor():
    hv = _bits([[[3.0, 4.0, 0.0, 0.0], [0.0, 0.0, 0.0, 0.0], [0.5, 0.5, 0.5, 0.5],
                 [-8.0, 0.0, 0.0, 0.0]]])
    r = oracle.hv_inv_norm(hv)
    np.testing.assert_allclose(r[0], [0.2, 1e8, 1.0, 0.125], rtol=1e-15)


def test_inverse_norms_match_a_library_norm():
    hv = synth.normal_bf16((21, 0), (2, 37, 48), 1.0)
    ref = 1.0 / torch.linalg.vector_norm(torch.from_numpy(synth.bf16_bits_to_f32(hv)).double(),
                                         dim=-1).numpy()
    np.testing.assert_allclose(oracle.hv_inv_norm(hv), ref, rtol=1e-14)


def test_prepared_relevance_hand_case():
    # the hand case of Eq. 8 with the inverse norms 1, 1, 1/sqrt2, 1 passed in
    hd = _bits([[[1.0, 0.0]]])
    hv = _bits([[[1.0, 0.0], [0.0, 1.0], [1.0, 1.0], [-1.0, 0.0]]])
    r = np.array([[1.0, 1.0, np.sqrt(0.5), 1.0]], np.float32)
    rel, cos = oracle.visual_relevance(hd, hv, [4], 2, return_cos=True, hv_inv_norm=r)
    np.testing.assert_allclose(cos[0, 0], [1.0, 0.0, float(np.float32(np.sqrt(0.5))), -1.0],
                               atol=1e-15)
    assert abs(rel[0, 0] - (1 + float(np.float32(np.sqrt(0.5)))) / 2) < 1e-15
    # a wrong inverse norm shows: the given values are used, not recomputed
    r2 = r.copy()
    r2[0, 1:] = 0.0
    assert oracle.visual_relevance(hd, hv, [4], 4, hv_inv_norm=r2)[0, 0] == 0.25


def test_prepared_relevance_is_eq8_when_norms_are_powers_of_two():
    # visual rows with exactly representable inverse norms (one non-zero element +-2^k): passing
    # the prepared inverse norms must give O2 bit for bit (scaling by 2^-k commutes with every
    # rounding)
    rng = np.random.default_rng(22)
    B, gamma, lv, d = 2, 3, 40, 16
    hv32 = np.zeros((B, lv, d), np.float32)
    pos = rng.integers(0, d, (B, lv))
    val = np.ldexp(rng.choice([-1.0, 1.0], (B, lv)), rng.integers(-6, 7, (B, lv)))
    for b in range(B):
        hv32[b, np.arange(lv), pos[b]] = val[b]
    hv = _bits(hv32)
    hd = synth.normal_bf16((22, 1), (B, gamma, d), 1.0)
    r = oracle.hv_inv_norm(hv)
    assert np.all(r == r.astype(np.float32))
    for n in (1, 5, 40):
        a = oracle.visual_relevance(hd, hv, [lv, lv - 7], n)
        b_ = oracle.visual_relevance(hd, hv, [lv, lv - 7], n, hv_inv_norm=r)
        np.testing.assert_array_equal(a, b_)


@pytest.mark.parametrize("seed,B,gamma,lv,d,N", [(31, 2, 3, 40, 24, 10), (32, 1, 5, 17, 64, 1)])
def test_prepared_relevance_matches_eq8_up_to_the_rounding_of_the_norms(seed, B, gamma, lv, d, N):
    hd = synth.normal_bf16((seed, 0), (B, gamma, d), 1.0)
    hv = synth.normal_bf16((seed, 1), (B, lv, d), 1.0)
    r = oracle.hv_inv_norm(hv)
    a, ca = oracle.visual_relevance(hd, hv, [lv] * B, N, return_cos=True)
    b_, cb = oracle.visual_relevance(hd, hv, [lv] * B, N, return_cos=True, hv_inv_norm=r)
    # binary32 inverse norms: half an ulp of relative error per cosine, nothing else
    np.testing.assert_allclose(cb, ca, rtol=6.1e-8, atol=1e-16)
    np.testing.assert_allclose(b_, a, rtol=6.1e-8, atol=1e-16)
    ref = torch.topk(torch.from_numpy(cb), N, dim=-1).values.mean(-1).numpy()
    np.testing.assert_allclose(b_, ref, rtol=1e-13, atol=1e-15)
