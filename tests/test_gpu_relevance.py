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
