"""Pins for oracle O7 (KV cache after a verified step): hand-derived row movements, and the
property that makes it the history of Eq. 1: attention over the committed cache equals attention
over a cache built directly from the context and the accepted tokens."""
import numpy as np
import pytest

import oracle
from golden_io import commit_cases
from paper_2604_05650_amd import synth

CASES = commit_cases()


def _labelled(cap, layers=2, Hkv=2, D=4):
    # k[l, 0, h, r, :] = label r (+ offsets that tell layers, heads and tensors apart)
    r = np.arange(cap, dtype=np.int32)
    k = np.zeros((layers, 1, Hkv, cap, D), np.int32)
    k += r[None, None, None, :, None]
    k += 1000 * np.arange(layers)[:, None, None, None, None]
    k += 100 * np.arange(Hkv)[None, None, :, None, None]
    return k, k + 50000


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_hand_derived_cases(case):
    k, v = _labelled(case["cap"])
    bb = np.array([case["kept"]], np.int32)
    k2, v2, new_len = oracle.kv_commit(k, v, np.array([case["ctx"]], np.int32), case["accept_len"],
                                       case["chain_len"], best_branch=bb,
                                       n_branches=case["n_branches"])
    assert new_len.tolist() == [case["new_len"]]
    for layer in range(2):
        for h in range(2):
            np.testing.assert_array_equal(k2[layer, 0, h, :, 0] - 1000 * layer - 100 * h,
                                          case["rows"])
            np.testing.assert_array_equal(v2[layer, 0, h, :, 1] - 1000 * layer - 100 * h - 50000,
                                          case["rows"])
    # the inputs are not modified
    np.testing.assert_array_equal(k, _labelled(case["cap"])[0])


def test_committed_cache_is_the_next_step_history():
    """Next-step attention (oracle O1) over the committed cache with the new lengths equals
    attention over a cache assembled directly from context + accepted tokens of the kept chain."""
    B, Hq, Hkv, D, cap, K, nbr = 2, 4, 2, 128, 48, 3, 2
    ctx = np.array([17, 30], np.int32)
    k = synth.normal_bf16((501, 0), (B, Hkv, cap, D), 1.0)
    v = synth.normal_bf16((501, 1), (B, Hkv, cap, D), 1.0)
    accept_len = np.array([1, 3, 2, 0], np.int32)       # chains of sequence 0, then sequence 1
    best = np.array([1, 0], np.int32)
    k2, v2, new_len = oracle.kv_commit(k, v, ctx, accept_len, K, best_branch=best, n_branches=nbr)
    assert new_len.tolist() == [20, 32]
    # direct assembly, written without reference to the draft-area layout of the result
    kd, vd = np.zeros_like(k), np.zeros_like(v)
    for b in range(B):
        chain = int(best[b])
        tau = int(accept_len[b * nbr + chain])
        hist_k = [k[b, :, r] for r in range(ctx[b])]
        hist_v = [v[b, :, r] for r in range(ctx[b])]
        for i in range(tau):
            hist_k.append(k[b, :, ctx[b] + chain * K + i])
            hist_v.append(v[b, :, ctx[b] + chain * K + i])
        kd[b, :, :len(hist_k)] = np.stack(hist_k, 1)
        vd[b, :, :len(hist_v)] = np.stack(hist_v, 1)
    # one new query row per sequence whose own K/V row sits right behind the history
    q = synth.normal_bf16((501, 2), (B, 1, Hq, D), 1.0)
    row_k = synth.normal_bf16((501, 3), (B, Hkv, D), 1.0)
    row_v = synth.normal_bf16((501, 4), (B, Hkv, D), 1.0)
    for b in range(B):
        for t, td, row in ((k2, kd, row_k), (v2, vd, row_v)):
            t[b, :, new_len[b]] = row[b]
            td[b, :, new_len[b]] = row[b]
    out_c, lse_c, _ = oracle.verify_attn(q, k2, v2, new_len)
    out_d, lse_d, _ = oracle.verify_attn(q, kd, vd, new_len)
    np.testing.assert_array_equal(out_c, out_d)
    np.testing.assert_array_equal(lse_c, lse_d)
