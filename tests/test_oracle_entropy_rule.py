"""Pins for oracle O5e: the entropy-gated accept rules of the text-only loose methods the paper
compares against (gate alone; gate plus deferred window).  Hand cases, special cases that
reduce to exact matching, a closed form, monotonicity, brute force on tiny drafts."""
import itertools

import numpy as np
import pytest

import oracle
from golden_io import entropy_cases

CASES = entropy_cases()


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_hand_derived_cases(case):
    vd, tau, bonus = oracle.verdicts_entropy(case["d"], case["y"], case["h"], case["threshold"],
                                             case["window"])
    np.testing.assert_array_equal(vd, case["verdict"])
    assert (tau, bonus) == (case["tau"], case["bonus"])


def test_closed_gate_is_exact_matching():
    # a threshold no entropy exceeds leaves the standard exact-match scheme (ln V bounds entropy)
    rng = np.random.default_rng(31)
    for _ in range(300):
        g = int(rng.integers(1, 12))
        y = rng.integers(0, 4, g).astype(np.int32)
        d = rng.integers(0, 4, g).astype(np.int32)
        h = (rng.random(g) * 12).astype(np.float32)
        for w in (0, 1, 4):
            vd, tau, bonus = oracle.verdicts_entropy(d, y, h, 12.0, w)
            neq = np.nonzero(d != y)[0]
            want = int(neq[0]) if neq.size else g
            np.testing.assert_array_equal(vd, (d == y).astype(np.uint8))
            assert tau == want and bonus == (int(y[want]) if want < g else -1)
            mask = np.zeros(g, np.uint8)
            assert oracle.verdicts(d, y, mask, 0)[1] == tau      # same as the paper's rule at lambda = 0


def test_open_gate_without_window_accepts_everything():
    rng = np.random.default_rng(32)
    for _ in range(100):
        g = int(rng.integers(1, 12))
        y = rng.integers(0, 4, g).astype(np.int32)
        d = rng.integers(0, 4, g).astype(np.int32)
        h = rng.random(g).astype(np.float32)
        vd, tau, bonus = oracle.verdicts_entropy(d, y, h, -1.0, 0)
        np.testing.assert_array_equal(vd, np.where(d == y, 1, 4))
        assert tau == g and bonus == -1


def test_gate_only_effective_rate_closed_form():
    # iid matches w.p. alpha, iid gate passes w.p. q: a position is accepted w.p.
    # alpha + (1 - alpha) q and the accepted length is the geometric sum of Prop. 2.2
    K, trials, alpha, q = 10, 100000, 0.6, 0.35
    rng = np.random.default_rng(33)
    y = np.arange(K, dtype=np.int32)
    taus = np.empty(trials)
    for t in range(trials):
        d = np.where(rng.random(K) < alpha, y, -1).astype(np.int32)
        h = np.where(rng.random(K) < q, 0.75, 0.125).astype(np.float32)
        taus[t] = oracle.verdicts_entropy(d, y, h, 0.5, 0)[1]
    ae = alpha + (1 - alpha) * q
    closed = ae * (1 - ae ** K) / (1 - ae)
    assert abs(taus.mean() - closed) < 4 * taus.std() / np.sqrt(trials)


def test_monotone_in_threshold_and_window():
    rng = np.random.default_rng(34)
    for _ in range(300):
        g = int(rng.integers(2, 11))
        y = rng.integers(0, 3, g).astype(np.int32)
        d = rng.integers(0, 3, g).astype(np.int32)
        h = rng.random(g).astype(np.float32)
        prev = g + 1
        for w in range(0, g + 1):          # a longer window can only reject more
            tau = oracle.verdicts_entropy(d, y, h, 0.3, w)[1]
            assert tau <= prev
            prev = tau
        prev = g + 1
        for th in (0.0, 0.2, 0.4, 0.6, 0.8, 1.0):    # a higher threshold too
            tau = oracle.verdicts_entropy(d, y, h, th, 1)[1]
            assert tau <= prev
            prev = tau


def test_window_brute_force_on_tiny_drafts():
    # every match pattern and gate pattern of up to five positions, windows 0..3: a mismatch is
    # accepted iff its gate is open and the set of window positions lies inside the set of
    # exactly matching draft positions
    for g in range(1, 6):
        y = np.arange(10, 10 + g, dtype=np.int32)
        for match in itertools.product((0, 1), repeat=g):
            d = np.where(np.array(match) == 1, y, 99).astype(np.int32)
            exact = {i for i in range(g) if match[i]}
            for gate in itertools.product((0, 1), repeat=g):
                h = np.where(np.array(gate) == 1, 0.5, 0.0625).astype(np.float32)
                for w in range(0, 4):
                    vd, tau, _ = oracle.verdicts_entropy(d, y, h, 0.25, w)
                    for i in range(g):
                        if match[i]:
                            want = 1
                        elif gate[i] and set(range(i + 1, i + w + 1)) <= exact:
                            want = 4
                        else:
                            want = 0
                        assert vd[i] == want, (match, gate, w, i)
                    lead = 0
                    while lead < g and vd[lead] != 0:
                        lead += 1
                    assert tau == lead


def test_chain_uses_the_rows_own_entropy():
    # O3 -> O5e: peaked rows (planted target direction, low entropy) stay strict, flat rows
    # (zero hidden state: uniform softmax, entropy ln V) pass the gate
    rng = np.random.default_rng(35)
    V, d = 64, 128
    from paper_2604_05650_amd import synth
    w = synth.f32_to_bf16_bits(rng.standard_normal((V, d)).astype(np.float32))
    wf = synth.bf16_bits_to_f32(w)
    h = np.zeros((1, 4, d), np.float32)
    h[0, 0] = 4.0 * wf[5]
    h[0, 2] = 4.0 * wf[9]
    hb = synth.f32_to_bf16_bits(h)
    draft = np.array([[6, 3, 9, 1]], np.int32)          # mismatch at 0 (peaked), 1 and 3 (flat)
    o = oracle.loose_accept(hb, w, draft, None, 0, 0, rule=oracle.RULE_ENTROPY_GATE,
                            entropy_threshold=0.2)
    assert o["target_ids"][0, 0] == 5 and o["target_ids"][0, 2] == 9
    assert o["entropy"][0, 0] < 0.2 and abs(o["entropy"][0, 1] - np.log(V)) < 1e-9
    np.testing.assert_array_equal(o["verdict"][0], [0, 4 if draft[0, 1] != o["target_ids"][0, 1] else 1, 1,
                                                    4 if draft[0, 3] != o["target_ids"][0, 3] else 1])
    assert o["accept_len"][0] == 0 and o["bonus_id"][0] == 5
    o2 = oracle.loose_accept(hb[:, 1:], w, draft[:, 1:], None, 0, 0,
                             rule=oracle.RULE_ENTROPY_WINDOW, entropy_threshold=0.2,
                             defer_window=1)
    # rows 1..3: flat (mismatch unless the uniform row's argmax 0 is drafted), peaked match, flat:
    # the first is confirmed by the match behind it, the last has no position behind it
    assert o2["verdict"][0].tolist() == [4, 1, 0] and o2["accept_len"][0] == 2
