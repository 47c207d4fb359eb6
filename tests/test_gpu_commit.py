"""GPU parity: lvspec_kv_commit against oracle O7, bit for bit (pure data movement)."""
import numpy as np
import pytest
import torch

import oracle
from golden_io import commit_cases
from paper_2604_05650_amd import synth
from parity import dev, t_bf16, t_i32

pytestmark = pytest.mark.gpu


def _bits(t):
    return synth.from_torch_bf16(t)


def _run(k, v, ctx, accept_len, K, best, nbr, tag):
    from paper_2604_05650_amd import binding as L
    print(f"[commit] {tag} k{k.shape} ctx{ctx.tolist()} K{K} br{nbr}", flush=True)
    kt, vt = t_bf16(k), t_bf16(v)
    new_len = L.kv_commit(kt, vt, t_i32(ctx), t_i32(accept_len), K,
                          best_branch=None if best is None else t_i32(best), n_branches=nbr)
    torch.cuda.synchronize()
    ko, vo, no = oracle.kv_commit(k, v, ctx, accept_len, K, best_branch=best, n_branches=nbr)
    np.testing.assert_array_equal(new_len.cpu().numpy(), no)
    np.testing.assert_array_equal(_bits(kt), ko)
    np.testing.assert_array_equal(_bits(vt), vo)
    return kt, vt, new_len


@pytest.mark.parametrize("case", commit_cases(), ids=[c["name"] for c in commit_cases()])
def test_hand_cases_through_the_library(case):
    cap, D, Hkv, layers = case["cap"], 128, 2, 2
    k = synth.normal_bf16((601, cap, 0), (layers, 1, Hkv, cap, D), 1.0)
    v = synth.normal_bf16((601, cap, 1), (layers, 1, Hkv, cap, D), 1.0)
    kt, vt, new_len = _run(k, v, np.array([case["ctx"]], np.int32), case["accept_len"],
                           case["chain_len"], np.array([case["kept"]], np.int32),
                           case["n_branches"], case["name"])
    assert new_len.tolist() == [case["new_len"]]
    np.testing.assert_array_equal(_bits(kt)[:, 0], k[:, 0][:, :, case["rows"]])
    np.testing.assert_array_equal(_bits(vt)[:, 0], v[:, 0][:, :, case["rows"]])


@pytest.mark.parametrize("layers,B,Hkv,D,cap,K,nbr", [
    (1, 1, 1, 8, 16, 1, 1), (3, 4, 2, 128, 200, 10, 2), (2, 3, 8, 128, 97, 4, 8),
    (1, 5, 4, 64, 64, 16, 2), (4, 2, 8, 128, 300, 5, 1), (2, 7, 3, 256, 50, 3, 3)])
def test_random_steps(layers, B, Hkv, D, cap, K, nbr):
    rng = np.random.default_rng((602, layers, B, K, nbr))
    k = synth.normal_bf16((602, layers, B, 0), (layers, B, Hkv, cap, D), 1.0)
    v = synth.normal_bf16((602, layers, B, 1), (layers, B, Hkv, cap, D), 1.0)
    ctx = rng.integers(0, cap - nbr * K + 1, B).astype(np.int32)
    ctx[0] = cap - nbr * K                      # a full cache
    accept_len = rng.integers(0, K + 1, B * nbr).astype(np.int32)
    accept_len[-1] = K
    best = rng.integers(0, nbr, B).astype(np.int32) if nbr > 1 else None
    if nbr > 1:
        best[-1] = nbr - 1
    _run(k, v, ctx, accept_len, K, best, nbr, "random")


def test_single_layer_strided_views_and_chain_mode_moves_nothing():
    from paper_2604_05650_amd import binding as L
    B, Hkv, cap, D, K = 2, 4, 40, 128, 5
    big = t_bf16(synth.normal_bf16((603, 0), (2, B, Hkv, cap + 8, D), 1.0))
    k, v = big[0, :, :, :cap], big[1, :, :, :cap]        # row stride D, head stride (cap+8)*D
    before = _bits(big).copy()
    ctx, tau = t_i32(np.array([7, 30])), t_i32(np.array([5, 2]))
    new_len = L.kv_commit(k, v, ctx, tau, K)
    torch.cuda.synchronize()
    assert new_len.tolist() == [12, 32]
    np.testing.assert_array_equal(_bits(big), before)
    # a tree on the same views: the second chain of sequence 1 kept
    ctx = t_i32(np.array([7, 20]))
    new_len = L.kv_commit(k, v, ctx, t_i32(np.array([3, 1, 0, 4])), K,
                          best_branch=t_i32(np.array([0, 1])), n_branches=2)
    torch.cuda.synchronize()
    assert new_len.tolist() == [10, 24]
    after = _bits(big)
    expect = before.copy()
    expect[:, 1, :, 20:24] = before[:, 1, :, 25:29]
    np.testing.assert_array_equal(after, expect)


def test_out_of_range_device_values_move_nothing():
    """Branch ids and lengths come from device memory: values outside their ranges are clamped,
    and a context that leaves no room for the draft rows moves no rows."""
    from paper_2604_05650_amd import binding as L
    B, Hkv, cap, D, K, nbr = 3, 2, 32, 128, 4, 2
    k = t_bf16(synth.normal_bf16((604, 0), (B, Hkv, cap, D), 1.0))
    v = t_bf16(synth.normal_bf16((604, 1), (B, Hkv, cap, D), 1.0))
    kb, vb = _bits(k).copy(), _bits(v).copy()
    ctx = t_i32(np.array([30, 5, 5]))                    # 30 + 8 > cap
    best = t_i32(np.array([1, 7, -3]))                   # 7 -> 1, -3 -> 0
    tau = t_i32(np.array([2, 2, 0, 9, 1, 0]))            # 9 -> 4
    new_len = L.kv_commit(k, v, ctx, tau, K, best_branch=best, n_branches=nbr)
    torch.cuda.synchronize()
    assert new_len.tolist() == [32, 9, 6]
    ek, ev = kb.copy(), vb.copy()
    ek[1, :, 5:9] = kb[1, :, 9:13]
    ev[1, :, 5:9] = vb[1, :, 9:13]
    np.testing.assert_array_equal(_bits(k), ek)
    np.testing.assert_array_equal(_bits(v), ev)


def test_tree_step_end_to_end_config1t():
    """Tree verify step on the small tree config: accept on the GPU, commit the kept chain, then
    the next step's attention over the committed cache matches the oracle chain (O5/O6 -> O7 -> O1)."""
    from paper_2604_05650_amd import binding as L
    cfg = synth.CONFIGS["c1t"]
    a = synth.attn_inputs(cfg)
    nbr, K = cfg.n_branches, cfg.gamma // cfg.n_branches
    chains = cfg.B * nbr
    rng = np.random.default_rng((605,))
    tau = rng.integers(0, K + 1, chains).astype(np.int32)
    best = np.array([oracle.select_branch(tau[s * nbr:(s + 1) * nbr]) for s in range(cfg.B)],
                    np.int32)
    kt, vt = t_bf16(a["k"]), t_bf16(a["v"])
    new_len = L.kv_commit(kt, vt, t_i32(a["kv_len"]), t_i32(tau), K, best_branch=t_i32(best),
                          n_branches=nbr)
    ko, vo, no = oracle.kv_commit(a["k"], a["v"], a["kv_len"], tau, K, best_branch=best,
                                  n_branches=nbr)
    np.testing.assert_array_equal(new_len.cpu().numpy(), no)
    # next step: one chain of K fresh draft rows behind the committed history
    cfg2 = cfg.with_(n_branches=1, gamma=K, seed=cfg.seed + 1)
    a2 = synth.attn_inputs(cfg2)
    q = a2["q"]
    for b in range(cfg.B):
        ko[b, :, no[b]:no[b] + K] = a2["k"][b, :, a2["kv_len"][b]:a2["kv_len"][b] + K]
        vo[b, :, no[b]:no[b] + K] = a2["v"][b, :, a2["kv_len"][b]:a2["kv_len"][b] + K]
    kt.copy_(t_bf16(ko)); vt.copy_(t_bf16(vo))
    out = L.verify_attn(t_bf16(q), kt, vt, new_len)
    torch.cuda.synchronize()
    o_out, _, _ = oracle.verify_attn(q, ko, vo, no)
    g = out.float().cpu().numpy().astype(np.float64)
    err = np.abs(g - o_out).max(-1) / np.maximum(np.abs(o_out).max(-1), 1e-30)
    assert err.max() <= 1e-2, err.max()
