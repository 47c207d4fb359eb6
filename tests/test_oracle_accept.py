"""Pins for oracle O4/O5 (Eq. 9, 10, 11, 2): hand cases, exact-match recovery, closed form."""
import numpy as np
import pytest

import oracle
from golden_io import accept_cases, paper_constants

CASES = accept_cases()


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_hand_derived_cases(case):
    mask, _ = oracle.loosened_set(case["a"], case["n_loose"])
    vd, tau, bonus = oracle.verdicts(case["d"], case["y"], mask, case["pst_window"])
    np.testing.assert_array_equal(vd, case["verdict"])
    assert (tau, bonus) == (case["tau"], case["bonus"])


def test_paper_constants():
    c = paper_constants()
    assert oracle.n_loose(0.7, 10) == c["n_loose_lambda0.7_K10"]
    # floor semantics of the slice 0:lambda*K for the draft lengths used in this repo
    assert [oracle.n_loose(0.7, g) for g in (3, 4, 5, 8, 10)] == [2, 2, 3, 5, 7]
    assert oracle.n_loose(0.0, 10) == 0 and oracle.n_loose(1.0, 10) == 10
    assert oracle.n_loose(0.3, 10) == 3 and oracle.n_loose(0.9, 10) == 9
    # tau counts accepted draft tokens out of K (the appendix's failure-rate arithmetic)
    assert abs((1 - c["tau_lvspec_32b"] / 10) - c["failure_rate_lvspec"]) < 5e-4
    assert abs((1 - c["tau_exact_chain_32b"] / 10) - c["failure_rate_exact"]) < 5e-4


def test_loosened_set_is_the_lowest_scores_stable():
    a = np.array([0.5, 0.1, 0.9, 0.1, 0.3], np.float32)
    mask, order = oracle.loosened_set(a, 3)
    np.testing.assert_array_equal(order, [1, 3, 4, 0, 2])
    np.testing.assert_array_equal(mask, [0, 1, 0, 1, 1])
    assert oracle.loosened_set(a, 0)[0].sum() == 0
    assert oracle.loosened_set(a, 5)[0].sum() == 5
    rng = np.random.default_rng(3)
    for _ in range(200):
        g = int(rng.integers(1, 17))
        a = rng.integers(0, 5, g).astype(np.float32)      # many ties
        n = int(rng.integers(0, g + 1))
        mask, order = oracle.loosened_set(a, n)
        np.testing.assert_array_equal(order, np.argsort(a, kind="stable"))
        assert mask.sum() == n


def test_lambda_zero_recovers_exact_match():
    # paper: decreasing lambda eventually recovers the standard exact-match scheme
    rng = np.random.default_rng(11)
    for _ in range(500):
        g = int(rng.integers(1, 12))
        y = rng.integers(0, 4, g).astype(np.int32)
        d = rng.integers(0, 4, g).astype(np.int32)
        a = rng.random(g).astype(np.float32)
        mask, _ = oracle.loosened_set(a, 0)
        vd, tau, bonus = oracle.verdicts(d, y, mask, 0)
        neq = np.nonzero(d != y)[0]
        want = int(neq[0]) if neq.size else g
        assert tau == want
        np.testing.assert_array_equal(vd, (d == y).astype(np.uint8))
        assert bonus == (int(y[want]) if want < g else -1)


def test_prefix_logic_single_reject_cuts():
    g = 8
    y = np.arange(100, 100 + g, dtype=np.int32)
    for j in range(g):
        d = y.copy()
        d[j] = 7
        vd, tau, bonus = oracle.verdicts(d, y, np.zeros(g, np.uint8), 0)
        assert tau == j and bonus == y[j] and vd.sum() == g - 1


@pytest.mark.parametrize("alpha,key", [(0.6, "strict_tau_alpha0.6_K10"),
                                       (0.8, "strict_tau_alpha0.8_K10")])
def test_strict_expected_length_closed_form(alpha, key):
    # Prop. 2.2: iid matches with probability alpha, K = 10
    K, trials = 10, 200000
    closed = alpha * (1 - alpha ** K) / (1 - alpha)
    assert abs(closed - paper_constants()[key]) < 1e-6
    rng = np.random.default_rng(2604)
    match = rng.random((trials, K)) < alpha
    y = np.arange(K, dtype=np.int32)
    zero = np.zeros(K, np.uint8)
    taus = np.empty(trials)
    for t in range(trials):
        d = np.where(match[t], y, -1).astype(np.int32)
        taus[t] = oracle.verdicts(d, y, zero, 0)[1]
    sigma = taus.std() / np.sqrt(trials)
    assert abs(taus.mean() - closed) < 4 * sigma


def test_loose_effective_rate_thm_2_3():
    # Thm 2.3's premise: if each position is loosened independently w.p. (1-rho), the effective
    # alignment rate is 1 - rho(1-alpha) and E[tau] = sum alpha_eff^k
    K, trials, alpha, rho = 10, 100000, 0.5, 0.3
    rng = np.random.default_rng(5)
    y = np.arange(K, dtype=np.int32)
    taus = np.empty(trials)
    for t in range(trials):
        d = np.where(rng.random(K) < alpha, y, -1).astype(np.int32)
        loose = (rng.random(K) < 1 - rho).astype(np.uint8)
        taus[t] = oracle.verdicts(d, y, loose, 0)[1]
    ae = 1 - rho * (1 - alpha)
    closed = ae * (1 - ae ** K) / (1 - ae)
    assert abs(taus.mean() - closed) < 4 * taus.std() / np.sqrt(trials)


def test_monotone_in_n_loose_and_window():
    rng = np.random.default_rng(17)
    for _ in range(300):
        g = int(rng.integers(2, 11))
        y = rng.integers(0, 6, g).astype(np.int32)
        d = rng.integers(0, 6, g).astype(np.int32)
        a = rng.random(g).astype(np.float32)
        prev = -1
        for n in range(g + 1):
            tau = oracle.verdicts(d, y, oracle.loosened_set(a, n)[0], 0)[1]
            assert tau >= prev
            prev = tau
        prev = -1
        for w in range(g + 1):
            tau = oracle.verdicts(d, y, np.zeros(g, np.uint8), w)[1]
            assert tau >= prev
            prev = tau
        # windows of gamma-1 and beyond are the whole draft
        a1 = oracle.verdicts(d, y, np.zeros(g, np.uint8), g - 1)
        a2 = oracle.verdicts(d, y, np.zeros(g, np.uint8), g + 5)
        np.testing.assert_array_equal(a1[0], a2[0])


def test_pst_brute_force_membership():
    # Eq. 11 with the whole draft as range: verdict 3 iff target token is in the draft set
    rng = np.random.default_rng(23)
    for _ in range(300):
        g = int(rng.integers(1, 9))
        y = rng.integers(0, 5, g).astype(np.int32)
        d = rng.integers(0, 5, g).astype(np.int32)
        vd, _, _ = oracle.verdicts(d, y, np.zeros(g, np.uint8), g)
        for i in range(g):
            want = 1 if d[i] == y[i] else (3 if y[i] in set(d.tolist()) else 0)
            assert vd[i] == want


def test_gate_only_restricts_loose():
    y = np.array([1, 2, 3], np.int32)
    d = np.array([9, 9, 3], np.int32)
    vd, tau, _ = oracle.verdicts(d, y, [1, 1, 0], 0, gate_ok=[1, 0, 1])
    np.testing.assert_array_equal(vd, [2, 0, 1])
    assert tau == 1
