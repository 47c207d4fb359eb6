"""GPU parity: lvspec_visual_relevance against oracle O2 (Eq. 8)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_05650_amd import synth
from parity import assert_scalars_close, dev, t_bf16, t_i32

pytestmark = pytest.mark.gpu


def _run(h_d, h_v, l_v, top_n):
    from paper_2604_05650_amd import binding as L
    rel = L.visual_relevance(t_bf16(h_d), t_bf16(h_v), t_i32(l_v), top_n)
    torch.cuda.synchronize()
    return rel.cpu().numpy().astype(np.float64)


def _check(h_d, h_v, l_v, top_n, tag):
    print(f"[rel] {tag} h_d{h_d.shape} h_v{h_v.shape} l_v{list(l_v)} N{top_n}", flush=True)
    g = _run(h_d, h_v, l_v, top_n)
    o = oracle.visual_relevance(h_d, h_v, l_v, top_n)
    e = assert_scalars_close(g, o, f"relevance {tag}")
    print(f"[rel] {tag} ok: {e:.2e}", flush=True)
    return g, o


@pytest.mark.parametrize("variant", ["literal", "structured"])
def test_config1(variant):
    cfg = synth.CONFIGS["c1"]
    h = synth.hidden_inputs(cfg, variant)
    g, o = _check(h["h_d"], h["h_v"], h["l_v"], cfg.top_n, f"c1 {variant}")
    if variant == "structured":
        # anchors and fillers are well separated: the ascending order must agree exactly
        np.testing.assert_array_equal(np.argsort(g[0], kind="stable"),
                                      np.argsort(o[0], kind="stable"))


@pytest.mark.parametrize("lv,d,N", [(1, 128, 1), (5, 128, 10), (63, 256, 10), (64, 256, 1),
                                    (65, 384, 64), (200, 1024, 100), (1000, 640, 1000),
                                    (777, 2048, 10),
                                    # more than 65536 video rows: slices of two and three
                                    # 1024-row chunks (N <= 16), radix-based selection (N = 40)
                                    (70000, 128, 10), (70000, 128, 40), (140000, 128, 16),
                                    (131072, 128, 1),
                                    # more rows than the sliced selection takes: one-kernel path
                                    (1100000, 128, 10)])
def test_ragged_sizes(lv, d, N):
    B, gamma = 1, 5
    h_d = synth.normal_bf16((201, lv, d, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((201, lv, d, 1), (B, lv + 3, d), 1.0)
    _check(h_d, h_v, [lv], N, f"lv{lv} d{d} N{N}")


@pytest.mark.parametrize("gamma", [1, 4, 8, 16])
def test_batch_with_different_visual_lengths(gamma):
    B, d, lv_max = 4, 512, 300
    h_d = synth.normal_bf16((202, gamma, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((202, gamma, 1), (B, lv_max, d), 1.0)
    _check(h_d, h_v, [300, 0, 129, 7], 10, f"batch g{gamma}")


def test_duplicates_and_scaled_rows():
    # many identical visual rows: the N-th largest value is tied; duplicates count by value.
    # rows scaled by powers of two keep their cosines.
    B, gamma, d, lv = 1, 3, 256, 150
    h_d = synth.normal_bf16((203, 0), (B, gamma, d), 1.0)
    base = synth.normal_bf16((203, 1), (B, 10, d), 1.0)
    h_v = np.tile(base, (1, 15, 1))
    h_v32 = synth.bf16_bits_to_f32(h_v) * np.float32(2.0) ** np.arange(lv)[None, :, None].clip(0, 6)
    h_v = synth.f32_to_bf16_bits(h_v32)
    _check(h_d, h_v, [lv], 20, "duplicates")


def test_long_rows_ragged_batch():
    # slices of two chunks; the second sequence ends inside the first slice, the third is empty
    B, gamma, d, lv_max = 3, 4, 128, 70001
    h_d = synth.normal_bf16((207, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((207, 1), (B, lv_max, d), 1.0)
    _check(h_d, h_v, [lv_max, 1500, 0], 10, "long ragged")


@pytest.mark.parametrize("lv,N", [(1000, 10), (5000, 10), (5000, 100), (300, 16), (70000, 10)])
def test_all_video_rows_identical(lv, N):
    # every cosine of a draft row is the same value: the selection's bound is tied with the
    # whole row (more candidates than either fast path holds), the answer is that value
    B, gamma, d = 1, 3, 256
    h_d = synth.normal_bf16((206, lv, 0), (B, gamma, d), 1.0)
    one = synth.normal_bf16((206, lv, 1), (B, 1, d), 1.0)
    h_v = np.tile(one, (1, lv, 1))
    g, o = _check(h_d, h_v, [lv], N, f"identical lv{lv} N{N}")
    cos = oracle.visual_relevance(h_d, h_v[:, :1], [1], 1)
    np.testing.assert_allclose(o, cos, rtol=1e-12)


def test_zero_rows():
    B, gamma, d, lv = 1, 2, 128, 70
    h_d = synth.normal_bf16((204, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((204, 1), (B, lv, d), 1.0)
    h_v[0, 3] = 0
    h_d[0, 1] = 0
    _check(h_d, h_v, [lv], 10, "zero rows")


def test_strided_rows():
    from paper_2604_05650_amd import binding as L
    B, gamma, d, lv = 2, 4, 256, 100
    h_d = synth.normal_bf16((205, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((205, 1), (B, lv, d), 1.0)
    big = torch.zeros((B, lv, 2 * d), dtype=torch.bfloat16, device=dev())
    big[..., :d] = t_bf16(h_v)
    rel = L.visual_relevance(t_bf16(h_d), big[..., :d], t_i32([lv, 50]), 10)
    torch.cuda.synchronize()
    o = oracle.visual_relevance(h_d, h_v, [lv, 50], 10)
    assert_scalars_close(rel.cpu().numpy(), o, "strided")


@pytest.mark.parametrize("name", ["c2", "c3", "c5"])
def test_full_size(name):
    from paper_2604_05650_amd import binding as L
    cfg = synth.CONFIGS[name]
    h = synth.hidden_inputs(cfg, "structured", device=dev())
    print(f"[rel] {name} launching", flush=True)
    rel = L.visual_relevance(h["h_d"], h["h_v"], t_i32(h["l_v"]), cfg.top_n)
    torch.cuda.synchronize()
    g = rel.cpu().numpy().astype(np.float64)
    hd, hv = synth.from_torch_bf16(h["h_d"]), synth.from_torch_bf16(h["h_v"])
    if name == "c5":     # the oracle covers two of the four sequences
        sel = [0, cfg.B - 1]
        o = oracle.visual_relevance(hd[sel], hv[sel], h["l_v"][sel], cfg.top_n)
        g = g[sel]
    else:
        o = oracle.visual_relevance(hd, hv, h["l_v"], cfg.top_n)
    e = assert_scalars_close(g, o, f"relevance {name}")
    print(f"[rel] {name} ok: {e:.2e}", flush=True)


# ---- prefill-side preparation (lvspec_hv_prepare) and relevance with prepared inverse norms ----
@pytest.mark.parametrize("B,lv,d", [(1, 1, 128), (2, 7, 256), (1, 1001, 384), (3, 130, 5120),
                                    (1, 66, 8192), (2, 4099, 1024)])
def test_hv_prepare_matches_the_oracle(B, lv, d):
    from paper_2604_05650_amd import binding as L
    h_v = synth.normal_bf16((208, B, lv, d), (B, lv, d), 1.0)
    h_v[0, lv // 2] = 0                                    # a zero row takes the norm floor
    h_v32 = synth.bf16_bits_to_f32(h_v)
    h_v32[-1, 0] *= 64.0                                   # and rows of very different scale
    h_v32[-1, lv - 1] *= 1.0 / 128.0
    h_v = synth.f32_to_bf16_bits(h_v32)
    print(f"[hv] prepare B{B} lv{lv} d{d}", flush=True)
    r = L.hv_prepare(t_bf16(h_v))
    torch.cuda.synchronize()
    o = oracle.hv_inv_norm(h_v)
    np.testing.assert_allclose(r.cpu().numpy().astype(np.float64), o, rtol=2e-6)


def test_hv_prepare_strided_rows():
    from paper_2604_05650_amd import binding as L
    B, lv, d = 2, 50, 256
    h_v = synth.normal_bf16((209, 0), (B, lv, d), 1.0)
    big = torch.zeros((B, lv + 5, 2 * d), dtype=torch.bfloat16, device=dev())
    big[:, :lv, :d] = t_bf16(h_v)
    r = L.hv_prepare(big[:, :lv, :d])
    torch.cuda.synchronize()
    np.testing.assert_allclose(r.cpu().numpy(), oracle.hv_inv_norm(h_v), rtol=2e-6)


def _check_prepared(h_d, h_v, l_v, top_n, tag):
    from paper_2604_05650_amd import binding as L
    print(f"[rel] prepared {tag} h_d{h_d.shape} h_v{h_v.shape} l_v{list(l_v)} N{top_n}", flush=True)
    tv = t_bf16(h_v)
    r = L.hv_prepare(tv)
    g = L.visual_relevance(t_bf16(h_d), tv, t_i32(l_v), top_n, hv_inv_norm=r)
    g0 = L.visual_relevance(t_bf16(h_d), tv, t_i32(l_v), top_n)
    torch.cuda.synchronize()
    g, g0 = g.cpu().numpy().astype(np.float64), g0.cpu().numpy().astype(np.float64)
    o = oracle.visual_relevance(h_d, h_v, l_v, top_n)                       # Eq. 8 itself
    o_given = oracle.visual_relevance(h_d, h_v, l_v, top_n, hv_inv_norm=r.cpu().numpy())
    assert_scalars_close(g, o, f"prepared relevance vs Eq. 8 {tag}")
    assert_scalars_close(g, o_given, f"prepared relevance vs given norms {tag}", tol=1e-4)
    # both ways of getting the norms agree far inside the tolerance
    assert_scalars_close(g, g0, f"prepared vs in-pass norms {tag}", tol=1e-4)


@pytest.mark.parametrize("lv,d,N,gamma", [(5, 128, 10, 3), (200, 1024, 100, 5), (777, 2048, 10, 8),
                                          (3000, 512, 10, 20), (70000, 128, 10, 5),
                                          (70000, 128, 40, 2), (1100000, 128, 10, 1)])
def test_prepared_relevance_ragged_sizes(lv, d, N, gamma):
    h_d = synth.normal_bf16((210, lv, d, 0), (1, gamma, d), 1.0)
    h_v = synth.normal_bf16((210, lv, d, 1), (1, lv + 3, d), 1.0)
    _check_prepared(h_d, h_v, [lv], N, f"lv{lv} d{d} N{N} g{gamma}")


def test_prepared_relevance_batch_and_zero_rows():
    B, gamma, d, lv_max = 4, 4, 512, 300
    h_d = synth.normal_bf16((211, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((211, 1), (B, lv_max, d), 1.0)
    h_v[0, 3] = 0
    h_d[2, 1] = 0
    _check_prepared(h_d, h_v, [300, 0, 129, 7], 10, "batch")


def test_given_inverse_norms_are_used_as_they_are():
    # inverse norms that are NOT those of h_v (all ones: relevance of raw dot products over
    # |h_d|): the library must follow its input, like the oracle with the same input
    from paper_2604_05650_amd import binding as L
    B, gamma, d, lv = 2, 5, 256, 500
    h_d = synth.normal_bf16((212, 0), (B, gamma, d), 1.0)
    h_v = synth.normal_bf16((212, 1), (B, lv, d), 0.25)
    ones = torch.ones((B, lv), dtype=torch.float32, device=dev())
    g = L.visual_relevance(t_bf16(h_d), t_bf16(h_v), t_i32([lv, 77]), 10, hv_inv_norm=ones)
    torch.cuda.synchronize()
    o = oracle.visual_relevance(h_d, h_v, [lv, 77], 10, hv_inv_norm=np.ones((B, lv), np.float32))
    assert_scalars_close(g.cpu().numpy(), o, "given norms")
    plain = oracle.visual_relevance(h_d, h_v, [lv, 77], 10)
    assert np.abs(o - plain).min() > 0.1       # the two really differ here


@pytest.mark.parametrize("name", ["c2", "c3", "c5"])
def test_prepared_full_size(name):
    from paper_2604_05650_amd import binding as L
    cfg = synth.CONFIGS[name]
    h = synth.hidden_inputs(cfg, "structured", device=dev())
    print(f"[rel] prepared {name} launching", flush=True)
    r = L.hv_prepare(h["h_v"])
    rel = L.visual_relevance(h["h_d"], h["h_v"], t_i32(h["l_v"]), cfg.top_n, hv_inv_norm=r)
    rel0 = L.visual_relevance(h["h_d"], h["h_v"], t_i32(h["l_v"]), cfg.top_n)
    torch.cuda.synchronize()
    g = rel.cpu().numpy().astype(np.float64)
    assert_scalars_close(g, rel0.cpu().numpy(), f"{name} prepared vs in-pass", tol=1e-4)
    hd, hv = synth.from_torch_bf16(h["h_d"]), synth.from_torch_bf16(h["h_v"])
    # inverse norms of a seeded sample of rows against the oracle; relevance of one sequence
    rows = np.random.default_rng(8).integers(0, hv.shape[1], 2000)
    o_r = oracle.hv_inv_norm(hv[-1:, rows])
    np.testing.assert_allclose(r[-1].cpu().numpy()[rows], o_r[0], rtol=2e-6)
    sel = [cfg.B - 1]
    o = oracle.visual_relevance(hd[sel], hv[sel], h["l_v"][sel], cfg.top_n)
    e = assert_scalars_close(g[sel], o, f"prepared relevance {name}")
    print(f"[rel] prepared {name} ok: {e:.2e}", flush=True)
