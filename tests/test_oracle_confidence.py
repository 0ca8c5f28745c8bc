"""Pins for the oracle's confidence estimator and budget rule (Method, Eq. 1).

The paper prints no worked number for Eq. 1, so the pins are closed forms, a
brute-force evaluation with the math module, an independent library composition
(scipy) and invariants.  Each would fail for a dropped term, a wrong weight
order, log2-vs-ln entropy, a missing normalisation by log V, or a margin taken
from sorted logits in the wrong order.
"""
import math

import numpy as np
import pytest
from scipy.special import expit, log_softmax, logsumexp
from scipy.stats import entropy as scipy_entropy

from oracle import confkv_oracle as O


def test_uniform_logits_closed_form():
    # uniform: H_hat = 1, m = 0 -> sigmoid = 1/2, p1 = 1/V  =>  c = 0.15 + 0.3 / V
    for V in (2, 7, 50257, 128256, 152064):
        for level in (0.0, -3.25, 11.0):
            c = O.confidence(np.full(V, level, dtype=np.float32))
            assert abs(c - (0.15 + 0.3 / V)) < 1e-12
    H_hat, m, p1 = O.confidence_terms(np.zeros(50257, dtype=np.float32))
    assert abs(H_hat - 1.0) < 1e-12 and m == 0.0 and abs(p1 - 1 / 50257) < 1e-15


def test_one_hot_gives_maximal_confidence():
    x = np.full(1000, -1.0e4, dtype=np.float32)
    x[123] = 0.0
    assert abs(O.confidence(x) - 1.0) < 1e-12
    x = np.full(1000, -np.inf, dtype=np.float32)
    x[5] = 2.0
    assert O.confidence(x) == pytest.approx(1.0, abs=1e-15)


@pytest.mark.parametrize("k,V", [(2, 10), (3, 1000), (17, 50257)])
def test_k_equal_maxima_closed_form(k, V):
    # k tokens share all the mass: H = log k, m = 0, p1 = 1/k
    x = np.full(V, -np.inf, dtype=np.float32)
    x[:k] = 1.5
    want = 0.4 * (1 - math.log(k) / math.log(V)) + 0.3 * 0.5 + 0.3 / k
    assert abs(O.confidence(x) - want) < 1e-12


@pytest.mark.parametrize("a,V", [(0.5, 11), (3.0, 5003), (9.0, 128256)])
def test_single_raised_logit_closed_form(a, V):
    x = np.zeros(V, dtype=np.float32)
    x[V // 3] = a
    Z = math.exp(a) + (V - 1)
    p1, po = math.exp(a) / Z, 1.0 / Z
    H = -(p1 * math.log(p1) + (V - 1) * po * math.log(po))
    want = 0.4 * (1 - H / math.log(V)) + 0.3 / (1 + math.exp(-a)) + 0.3 * p1
    H_hat, m, p_top = O.confidence_terms(x)
    assert abs(m - a) < 1e-12 and abs(p_top - p1) < 1e-14 and abs(H_hat - H / math.log(V)) < 1e-12
    assert abs(O.confidence(x) - want) < 1e-12


def test_brute_force_tiny_vocab():
    x = [0.3, -1.2, 2.0, 0.9]
    e = [math.exp(v) for v in x]
    Z = sum(e)
    p = sorted(v / Z for v in e)
    H = -sum(v * math.log(v) for v in p)
    m = math.log(p[-1]) - math.log(p[-2])
    want = 0.4 * (1 - H / math.log(4)) + 0.3 / (1 + math.exp(-m)) + 0.3 * p[-1]
    assert abs(O.confidence(np.array(x, dtype=np.float64)) - want) < 1e-12
    # weights are applied in the order (entropy, margin, top): perturb one at a time
    assert abs(O.confidence(np.array(x), (1.0, 0.0, 0.0)) - (1 - H / math.log(4))) < 1e-12
    assert abs(O.confidence(np.array(x), (0.0, 1.0, 0.0)) - 1 / (1 + math.exp(-m))) < 1e-12
    assert abs(O.confidence(np.array(x), (0.0, 0.0, 1.0)) - p[-1]) < 1e-12


@pytest.mark.parametrize("std", [0.5, 3.0, 6.0])
def test_matches_scipy_composition(std):
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(50257) * std).astype(np.float32)
    lp = log_softmax(x.astype(np.float64))
    H = scipy_entropy(np.exp(lp))
    top = np.partition(lp, -2)[-2:]
    m = top[1] - top[0]
    want = 0.4 * (1 - H / np.log(x.size)) + 0.3 * expit(m) + 0.3 * np.exp(top[1])
    assert abs(O.confidence(x) - want) < 1e-12
    assert abs(np.exp(top[1]) - np.exp(np.max(x.astype(np.float64)) - logsumexp(x.astype(np.float64)))) < 1e-15


def test_invariances_and_bounds():
    rng = np.random.default_rng(11)
    V = 4099
    x = (rng.standard_normal(V) * 4).astype(np.float64)
    c = O.confidence(x)
    assert abs(O.confidence(x + 37.5) - c) < 1e-12          # shift invariance
    assert abs(O.confidence(rng.permutation(x)) - c) < 1e-12  # permutation invariance
    assert 0.15 + 0.3 / V - 1e-12 <= c <= 1.0
    # sharper distribution -> more confident (monotone in temperature for this sample)
    assert O.confidence(2 * x) > c > O.confidence(0.5 * x)


def test_duplicate_maximum_counts_with_multiplicity():
    x = np.array([1.0, 5.0, 5.0, -2.0])
    _, m, _ = O.confidence_terms(x)
    assert m == 0.0


def test_budget_rule_truth_table():
    tau = float(np.float32(0.7))
    assert O.select_budget(tau, tau, 128, 256) == (True, 128)           # c >= tau is tight
    assert O.select_budget(np.nextafter(tau, 0), tau, 128, 256) == (False, 256)
    assert O.select_budget(0.99, tau, 128, 256) == (True, 128)
    assert O.select_budget(0.2, tau, 128, 256) == (False, 256)
    with pytest.raises(ValueError):
        O.select_budget(0.5, tau, 300, 256)                            # N_high <= N_low


def test_pyramid_geometric_schedule():
    # N(l) = max(N_min, N0 * beta^(l/L)); beta = 0.5, N_min = 96 (paper defaults)
    got = O.pyramid_geometric(256, 12)
    assert got == [256, 241, 228, 215, 203, 191, 181, 170, 161, 152, 143, 135]
    got = O.pyramid_geometric(128, 12)
    assert got[:6] == [128, 120, 114, 107, 101, 96] and all(v == 96 for v in got[5:])
    big = O.pyramid_geometric(4096, 64)
    assert big[0] == 4096 and all(a >= b for a, b in zip(big, big[1:]))
    assert big[32] == int(4096 * 0.5 ** 0.5)                            # half-way: N0 / sqrt(2)
    assert O.pyramid_geometric(100, 4, beta=0.5, n_min=96) == [100, 96, 96, 96]
