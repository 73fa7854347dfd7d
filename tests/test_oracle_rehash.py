"""Pins for the Step Rehash oracle: cosine closed forms, Algorithm 1 worked by hand."""
import math
import os

import numpy as np
import pytest

import oracle
import si_workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_cases.txt")


def _rule_matrix(rule, K):
    S = np.zeros((K, K))
    for i in range(K):
        for j in range(K):
            if rule.startswith("const:"):
                S[i, j] = float(rule.split(":")[1])
            elif rule == "identity":
                S[i, j] = 1.0 if i == j else 0.0
            elif rule.startswith("band:"):
                S[i, j] = 1.0 if abs(i - j) <= int(rule.split(":")[1]) else 0.0
            elif rule.startswith("linear:"):
                S[i, j] = 1.0 - float(rule.split(":")[1]) * abs(i - j)
    return S


def _golden_cases():
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, K, gamma, rule, G = [t.strip() for t in line.split("|")]
        yield name, int(K), float(gamma), rule, [int(t) for t in G.split()]


@pytest.mark.parametrize("name,K,gamma,rule,G", list(_golden_cases()))
def test_key_step_search_hand_worked(name, K, gamma, rule, G):
    assert oracle.key_step_search_ref(_rule_matrix(rule, K), gamma, K) == G


def test_key_step_search_uses_anchor_column_not_previous_step():
    # adjacent steps always similar, but drift against the anchor accumulates
    K = 9
    S = _rule_matrix("linear:0.02", K)       # S[i][i-1] = 0.98 everywhere
    G = oracle.key_step_search_ref(S, 0.95, K)
    assert G == [0, 3, 6, 8]                 # 1-0.02*3 = 0.94 < 0.95 at distance 3
    # asymmetric S: only the [i][anchor] entry is read
    S2 = np.ones((4, 4)); S2[2, 0] = 0.0
    assert oracle.key_step_search_ref(S2, 0.5, 4) == [0, 2, 3]
    S3 = np.ones((4, 4)); S3[0, 2] = 0.0
    assert oracle.key_step_search_ref(S3, 0.5, 4) == [0, 3]


def test_key_step_search_rejects_bad_arguments():
    S = np.ones((3, 3))
    for bad in (1.5, float("nan")):
        with pytest.raises(ValueError):
            oracle.key_step_search_ref(S, bad, 3)
    with pytest.raises(ValueError):
        oracle.key_step_search_ref(S, 0.5, 0)
    with pytest.raises(ValueError):
        oracle.key_step_search_ref(np.zeros((3, 3)), 0.5, 3)   # diagonal below threshold


def test_cosine_closed_forms():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(1000)
    assert oracle.cosine_ref(a, a) == pytest.approx(1.0, abs=1e-15)
    assert oracle.cosine_ref(a, -a) == pytest.approx(-1.0, abs=1e-15)
    assert oracle.cosine_ref(a, 3.7 * a) == pytest.approx(1.0, abs=1e-15)
    e0 = np.zeros(8); e0[0] = 2.0
    e3 = np.zeros(8); e3[3] = -5.0
    assert oracle.cosine_ref(e0, e3) == 0.0
    # 3-4-5: cos((1,0),(3,4)) = 0.6 ; 45 degrees
    assert oracle.cosine_ref([1.0, 0.0], [3.0, 4.0]) == pytest.approx(0.6, abs=1e-15)
    assert oracle.cosine_ref([1.0, 0.0], [1.0, 1.0]) == pytest.approx(1 / math.sqrt(2), abs=1e-15)
    # whole tensor flattened, shape ignored
    t = rng.standard_normal((2, 3, 4)); u = rng.standard_normal((2, 3, 4))
    assert oracle.cosine_ref(t, u) == pytest.approx(
        float((t * u).sum() / math.sqrt((t * t).sum() * (u * u).sum())), abs=1e-14)
    # degenerate cases
    z = np.zeros(5)
    assert oracle.cosine_ref(z, z) == 1.0 and oracle.cosine_ref(z, e0[:5]) == 0.0
    assert math.isnan(oracle.cosine_ref([1.0, float("inf")], [1.0, 1.0]))
    assert math.isnan(oracle.cosine_ref([1.0, float("nan")], [1.0, 1.0]))


def test_decision_rule_and_ties():
    a = np.array([1.0, 0.0]); b = np.array([3.0, 4.0])          # cos = 0.6
    assert oracle.rehash_decision_ref(a, b, 0.59) == 1
    assert oracle.rehash_decision_ref(a, b, 0.61) == 0
    x = np.random.default_rng(1).standard_normal(257)
    assert oracle.rehash_decision_ref(x, x, 1.0) == 1              # tie: cos == gamma -> reuse
    assert oracle.rehash_decision_ref(x, -x, -1.0) == 1
    assert oracle.rehash_decision_ref(x, -x, -0.99) == 0
    z = np.zeros(4)
    assert oracle.rehash_decision_ref(z, z, 0.95) == 1
    assert oracle.rehash_decision_ref(z, x[:4], 0.95) == 0
    assert oracle.rehash_decision_ref(z, x[:4], 0.0) == 1
    bad = x.copy(); bad[3] = float("nan")
    assert oracle.rehash_decision_ref(bad, x, -1.0) == 0
    assert oracle.rehash_decision_ref(x, x, float("nan")) == 0


def test_gaussian_drift_closed_form():
    """x_k = x_0 + sum of independent N(0, s_t^2): cos(x_0, x_k) -> 1/sqrt(1 + sum s_t^2)."""
    rng = np.random.default_rng(3)
    n = 400_000
    x0 = rng.standard_normal(n)
    xk = x0.copy()
    acc = 0.0
    for t in range(1, 6):
        s = wl.cfg5_sigma(t)
        xk = xk + s * rng.standard_normal(n)
        acc += s * s
        assert oracle.cosine_ref(x0, xk) == pytest.approx(1 / math.sqrt(1 + acc), abs=4e-3)


def test_replay_hands_back_cached_feature():
    calls = []

    def compute(t):
        calls.append(t)
        return np.full(3, float(t))

    got = list(oracle.rehash_replay_ref(compute, [0, 3, 5], 6))
    assert calls == [0, 3, 5]
    assert [int(f[0]) for _, f, _ in got] == [0, 0, 0, 3, 3, 5]
    assert [r for _, _, r in got] == [True, False, False, True, False, True]


def test_causal_walk_equals_algorithm1_on_the_input_map():
    """The one-pass rule recomputes exactly at Algorithm 1's key steps of the INPUT similarity map
    (its anchored walk), except that Algorithm 1 also forces the last step."""
    rng = np.random.default_rng(11)
    for trial in range(20):
        K = int(rng.integers(2, 12))
        n = 64
        xs = [rng.standard_normal(n)]
        for t in range(1, K):
            xs.append(xs[-1] + float(rng.uniform(0.05, 0.6)) * rng.standard_normal(n))
        gamma = float(rng.uniform(0.6, 0.99))
        S = np.array([[oracle.cosine_ref(xs[i], xs[j]) for j in range(K)] for i in range(K)])
        G = oracle.key_step_search_ref(S, float(np.float32(gamma)), K)
        got = list(oracle.rehash_causal_ref(xs, lambda x: 2.0 * x, gamma))
        rec = [t for t, _, r, _ in got if r]
        assert sorted(set(rec + [K - 1])) == G and rec[0] == 0
        # hand-back: a reused step returns the anchor's output, bit for bit
        anchor = None
        for t, y, r, c in got:
            if r:
                anchor = t
                assert np.array_equal(y, 2.0 * xs[t])
            else:
                assert np.array_equal(y, 2.0 * xs[anchor])
                assert c == oracle.cosine_ref(xs[t], xs[anchor]) and c >= np.float32(gamma) - 1e-15


def test_causal_walk_extremes_and_chaining():
    rng = np.random.default_rng(12)
    xs = [rng.standard_normal(32) for _ in range(5)]            # unrelated inputs: |cos| small
    calls = []

    def compute(x):
        calls.append(1)
        return x + 1.0

    assert [r for _, _, r, _ in oracle.rehash_causal_ref(xs, compute, 0.9)] == [True] * 5
    assert [r for _, _, r, _ in oracle.rehash_causal_ref(xs, compute, -1.0)] == [True] + [False] * 4
    same = [xs[0]] * 4                                           # identical inputs: cos = 1 >= gamma = 1 (tie reuses)
    assert [r for _, _, r, _ in oracle.rehash_causal_ref(same, compute, 1.0)] == [True, False, False, False]
    # chaining through a stack: a reused block hands its successor the anchor's output again, so the
    # successor's input repeats exactly and it reuses too
    drift = [xs[0], xs[0] + 0.01 * xs[1], xs[0] + 0.02 * xs[2], xs[3]]
    first = list(oracle.rehash_causal_ref(drift, lambda x: np.tanh(x), 0.95))
    second = list(oracle.rehash_causal_ref([y for _, y, _, _ in first], lambda x: x * x, 0.95))
    assert [r for _, _, r, _ in first] == [True, False, False, True]
    assert [r for _, _, r, _ in second] == [True, False, False, True]
    assert all(c == 1.0 or math.isnan(c) or r for _, _, r, c in second)


def test_causal_walk_cfg5_schedule_prediction():
    """Gaussian drift of the cfg5 schedule: cos(x_t, x_anchor) = 1/sqrt(1 + sum sigma^2) in the limit,
    which first falls below 0.95 four steps after an anchor at step 0 (0.981, 0.966, 0.956, 0.949)."""
    acc, pred = 0.0, []
    for t in range(1, 5):
        acc += wl.cfg5_sigma(t) ** 2
        pred.append(1 / math.sqrt(1 + acc))
    assert pred[2] > 0.95 > pred[3]
    rng = np.random.default_rng(13)
    n = 2_000_000                                                # margin at t = 4 is ~1e-3; sampling noise ~ 1/sqrt(n)
    xs = [rng.standard_normal(n)]
    for t in range(1, wl.CFG5_STEPS):
        xs.append(xs[-1] + wl.cfg5_sigma(t) * rng.standard_normal(n))
    rec = [t for t, _, r, _ in oracle.rehash_causal_ref(xs, lambda x: x, wl.CFG5_GAMMA) if r]
    assert rec[:2] == [0, 4]
