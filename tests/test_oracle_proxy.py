"""Pins of the proxy oracle (oracle/proxy_oracle.py) against what the paper and the mathematics
fix: the uniform case, closed forms for two-valued intervals, the Taylor relation between P_c and
the central moments, invariances, monotonicity in an outlier, and the decision rule."""
import math

import numpy as np
import pytest

from oracle import proxy_oracle as P


def test_equally_spaced_weights_give_zero():
    # Eq. "absolute_case": fixed intervals -> G' = 1/n -> P_c = 0; delta = 0 -> P_f = 0.
    W = np.arange(4097, dtype=np.float64) * 0.25 - 3.0
    rng = np.random.default_rng(0)
    W = rng.permutation(W).reshape(17, 241)         # sorting undoes any arrangement
    Pc, Pf = P.proxies(W)
    assert abs(Pc) < 1e-12 and abs(Pf) < 1e-9


def two_level(p, a, q, b):
    """Closed forms for intervals: p of length a and q of length b (written independently of the
    oracle: plain sums over the two distinct values)."""
    n = p + q
    S = p * a + q * b
    ga, gb = a / S, b / S
    H = -(p * ga * math.log(ga) + q * gb * math.log(gb))
    Pc = math.log(n) - H
    da, db = ga - 1.0 / n, gb - 1.0 / n
    Pf = 0.0
    for k in range(2, 6):
        Mk = (p * da ** k + q * db ** k) / n
        Pf += n ** k / (k * (k - 1)) * abs(Mk)
    return Pc, Pf


@pytest.mark.parametrize("p,a,q,b", [(100, 1.0, 100, 3.0), (999, 0.5, 1, 200.0), (7, 2.0, 50, 0.125),
                                     (100, 3.0, 5, 0.01)])   # the last one has negative odd moments
def test_two_valued_intervals_closed_form(p, a, q, b):
    gaps = np.array([a] * p + [b] * q)
    np.random.default_rng(1).shuffle(gaps)          # order of the intervals is irrelevant
    W = np.concatenate([[0.0], np.cumsum(gaps)])
    Pc, Pf = P.proxies(W)
    ePc, ePf = two_level(p, a, q, b)
    assert Pc == pytest.approx(ePc, rel=1e-10, abs=1e-13)
    assert Pf == pytest.approx(ePf, rel=1e-9)


def test_second_order_term_is_half_the_squared_coefficient_of_variation():
    # v_2 |M_2| = n^2/2 * var(G') = var(G / mean G) / 2
    rng = np.random.default_rng(2)
    W = rng.normal(size=5000)
    G = P.intervals(W)
    t = G / G.mean()
    assert P.fine(G, terms=2) == pytest.approx(0.5 * np.mean((t - 1.0) ** 2), rel=1e-10)


def test_taylor_relation_between_coarse_proxy_and_moments():
    # Eq. "taylor_final": for a small disturbance of the uniform intervals,
    # P_c = sum_{k>=2} (-1)^k n^(k-1)/(k(k-1)) sum_i delta_i^k + o(delta^K).
    rng = np.random.default_rng(3)
    n = 2000
    for eps, tol in ((0.05, 2e-9), (0.2, 3e-6)):
        gaps = 1.0 + eps * rng.uniform(-1, 1, n)
        W = np.concatenate([[0.0], np.cumsum(gaps)])
        G = P.intervals(W)
        delta = G / G.sum() - 1.0 / n
        series = sum((-1) ** k * n ** (k - 1) / (k * (k - 1)) * np.sum(delta ** k) for k in range(2, 7))
        Pc = P.coarse(G)
        assert Pc > 0
        assert abs(Pc - series) < tol, (eps, Pc, series)
        # leading term alone: relative error of order eps
        lead = n / 2.0 * np.sum(delta ** 2)
        assert abs(Pc - lead) / Pc < 1.5 * eps


def test_coarse_proxy_nonnegative_and_invariant():
    rng = np.random.default_rng(4)
    for _ in range(5):
        W = rng.standard_t(df=3, size=(64, 50))
        Pc, Pf = P.proxies(W)
        assert Pc >= 0 and Pf >= 0
        # positive scaling and shift leave G' unchanged
        Pc2, Pf2 = P.proxies(3.5 * W - 11.0)
        assert Pc2 == pytest.approx(Pc, rel=1e-9) and Pf2 == pytest.approx(Pf, rel=1e-7)
        # so does any rearrangement of the entries
        Pc3, Pf3 = P.proxies(rng.permutation(W.ravel()))
        assert Pc3 == Pc and Pf3 == Pf


def test_outlier_raises_the_fine_proxy_more_than_the_coarse_one():
    # The fine-grained proxy exists because a few outliers barely move the entropy gap.
    base = np.linspace(-1.0, 1.0, 20001)
    prev_c, prev_f = P.proxies(base)
    ratios = []
    for mag in (2.0, 4.0, 8.0, 16.0):
        W = np.concatenate([base, [mag]])
        Pc, Pf = P.proxies(W)
        assert Pc > prev_c and Pf > prev_f       # both grow with the outlier ...
        ratios.append(Pf / Pc)
        prev_c, prev_f = Pc, Pf
    assert all(b > a for a, b in zip(ratios, ratios[1:]))   # ... the fine one faster
    assert ratios[-1] > 1e3


def test_ties_and_constant_matrix():
    W = np.array([0.0, 0.0, 1.0, 1.0, 1.0, 2.0, 4.0, 4.0])
    # intervals 0,1,0,0,1,2,0 -> G' = 0,.25,0,0,.25,.5,0 ; n = 7
    H = -(0.25 * math.log(0.25) * 2 + 0.5 * math.log(0.5))
    assert P.proxies(W)[0] == pytest.approx(math.log(7) - H, rel=1e-12)
    d = np.array([0, .25, 0, 0, .25, .5, 0]) - 1 / 7
    ePf = sum(7 ** k / (k * (k - 1)) * abs(np.sum(d ** k) / 7) for k in range(2, 6))
    assert P.proxies(W)[1] == pytest.approx(ePf, rel=1e-12)
    assert P.proxies(np.full((4, 4), 2.5)) == (0.0, 0.0)


def test_decision_rule():
    # Eq. "multi_scale_proxy": SQ only if both proxies are below their thresholds.
    assert P.phi(1.0, 10.0, tau_c=1.5, tau_f=30.0) == 1
    assert P.phi(1.0, 30.0, tau_c=1.5, tau_f=30.0) == 0     # P_f >= tau_f
    assert P.phi(1.5, 10.0, tau_c=1.5, tau_f=30.0) == 0     # P_c >= tau_c
    assert P.phi(2.0, 99.0, tau_c=1.5, tau_f=30.0) == 0


def test_sixteen_bit_widening():
    bits = np.array([0x3C00, 0xC000, 0x0001, 0x8000], np.uint16)
    assert P.widen16(bits, "f16").tolist() == [1.0, -2.0, 2.0 ** -24, -0.0]
    bits = np.array([0x3F80, 0xC000, 0x0080], np.uint16)
    assert P.widen16(bits, "bf16").tolist() == [1.0, -2.0, 2.0 ** -126]
