"""Pins for the oracle's draft-tree step (appendix on draft token trees)."""
import numpy as np
import pytest

from oracle import lvspec_oracle as oracle
from tests.golden_io import tree_cases


def _chain_tau(c, n_loose, w):
    mask, _ = oracle.loosened_set(c["a"], n_loose)
    _, tau, _ = oracle.verdicts(c["d"], c["y"], mask, w)
    return tau


@pytest.mark.parametrize("case", tree_cases(), ids=lambda c: c["name"])
def test_hand_derived_tree_cases(case):
    taus = [_chain_tau(c, case["n_loose"], case["pst_window"]) for c in case["chains"]]
    assert taus == case["tau"].tolist()
    assert oracle.select_branch(taus) == case["kept"]


def test_kept_branch_is_first_maximum_brute_force():
    rng = np.random.default_rng(7)
    for _ in range(500):
        n = int(rng.integers(1, 9))
        tau = rng.integers(0, 11, size=n).astype(np.int32)
        kept = oracle.select_branch(tau)
        assert tau[kept] == tau.max()
        assert not (tau[:kept] == tau.max()).any()


def test_kept_length_never_below_any_single_chain():
    # the tree can only lengthen the accepted prefix of a step (the paper reports a larger tau
    # with the tree than without)
    rng = np.random.default_rng(11)
    for _ in range(200):
        tau = rng.integers(0, 11, size=2).astype(np.int32)
        assert tau[oracle.select_branch(tau)] >= tau[0]


def test_chain_composition_reports_branches():
    # two copies of the same chain through the chained entry: equal lengths, branch 0 kept;
    # breaking chain 0 at its first slot hands the step to chain 1
    from paper_2604_05650_amd import synth
    cfg = synth.CONFIGS["c1"]
    w = synth.lm_head(cfg)
    h = synth.hidden_inputs(cfg)["h_d"][:1]
    h2 = np.concatenate([h, h], axis=0)
    rel = np.tile(np.linspace(0.1, 0.9, cfg.gamma, dtype=np.float32), (2, 1))
    one = oracle.loose_accept(h, w, np.zeros((1, cfg.gamma), np.int32), rel[:1], 0, 0)
    y = one["target_ids"][0]
    d = np.stack([y, y]).astype(np.int32)
    out = oracle.loose_accept(h2, w, d, rel, 0, 0, n_branches=2)
    assert out["accept_len"].tolist() == [cfg.gamma, cfg.gamma] and out["best_branch"].tolist() == [0]
    d[0, 0] = (y[0] + 1) % cfg.V
    out = oracle.loose_accept(h2, w, d, rel, 0, 0, n_branches=2)
    assert out["accept_len"].tolist() == [0, cfg.gamma] and out["best_branch"].tolist() == [1]
