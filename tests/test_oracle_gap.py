"""Pins for the oracle's measured logit gap and the gap form of the temperature update
(Appendix A, the relation tau1 = tau0 (1 + tau0 ln(alpha) / Delta)) -- not gpu."""
import math

import numpy as np
import pytest

from oracle import e3_oracle as o

V_Q = 151_936


def _gap(z, tau=1.0):
    return o.logit_gaps(np.ascontiguousarray(z, np.float32).reshape(1, -1), None, tau)[0]


def test_two_level_model_returns_delta_for_any_tau():
    for delta in (0.5, 3.0, 15.0, 16.0, 17.0):
        row = np.zeros(V_Q, np.float32)
        row[777] = delta
        for tau in (0.3, 1.0, 2.0):
            assert _gap(row, tau) == pytest.approx(delta, rel=1e-10)   # 151,935 equal terms summed


def test_small_worked_rows():
    assert _gap([5.0, 2.0]) == pytest.approx(3.0)
    # z = (4, 3, 1): rest weights e^-1, e^-3 -> (1 e^-1 + 3 e^-3) / (e^-1 + e^-3)
    w1, w2 = math.exp(-1), math.exp(-3)
    assert _gap([4.0, 3.0, 1.0]) == pytest.approx((w1 + 3 * w2) / (w1 + w2), rel=1e-14)
    # tau = 1/2 doubles the exponents but not the gaps
    w1, w2 = math.exp(-2), math.exp(-6)
    assert _gap([4.0, 3.0, 1.0], 0.5) == pytest.approx((w1 + 3 * w2) / (w1 + w2), rel=1e-14)
    # a tie at the top: the second maximum belongs to the rest with gap 0
    assert _gap([2.0, 2.0]) == 0.0
    assert math.isnan(_gap([1.0]))
    # uniform rows: every gap is 0
    assert _gap(np.full(100, 1.5)) == 0.0


def test_invariances():
    rng = np.random.default_rng(0)
    z = (rng.normal(0, 2, 400) * 32).round() / 32
    g = _gap(z, 0.75)
    assert _gap(z + 8.0, 0.75) == pytest.approx(g, rel=1e-13)
    assert _gap(z * 2.0, 1.5) == pytest.approx(2 * g, rel=1e-13)       # gap is in logit units


def test_ties_entropy_through_the_decomposition():
    # Appendix A: H = beta sum_i p_i Delta_i + ln Z, and sum_i p_i Delta_i = (1 - p_max) Delta_hat
    rng = np.random.default_rng(1)
    for V, tau in ((7, 1.0), (300, 0.6), (5000, 1.4)):
        z = rng.normal(0, 3, V).astype(np.float32)
        t32 = float(np.float32(tau))
        lp = o.log_softmax_row(z, tau)
        H = o.logprob_entropy(z.reshape(1, -1), None, None, None, tau).entropy[0]
        p_max = math.exp(lp.max())
        lnZ = -lp.max()                                                   # Z relative to the maximum
        assert H == pytest.approx((1 - p_max) * _gap(z, tau) / t32 + lnZ, rel=1e-11)


def test_gap_update_values_and_relation_to_eq4():
    D = math.log(V_Q) + math.log(math.log(V_Q))
    # with Delta = ln|V| + ln ln|V| the gap form is Eq. 4
    for tau, alpha in ((1.0, 1.1), (1.2, 0.9), (0.6, 2.0)):
        rc, a, _ = o.temperature_update_gap(tau, 1.0, alpha, D)
        rc2, b, _ = o.temperature_update(tau, 1.0, alpha, V_Q)
        assert rc == 0 and rc2 == 0 and a == pytest.approx(b, rel=1e-15)
    assert o.temperature_update_gap(1.0, 1.0, math.e, 2.0)[1] == pytest.approx(1.5)
    assert o.temperature_update_gap(2.0, 0.5, 0.5, 7.0)[1] == 2.0             # alpha = 1
    rc, nxt, tgt = o.temperature_update_gap(1.0, 0.3, 0.4, 10.0, t=480, t_anneal=288, t_max=480, eta=0.9)
    assert rc == 0 and tgt == pytest.approx(0.36) and nxt == pytest.approx(1 + math.log(1.2) / 10)
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        assert o.temperature_update_gap(1.0, 0.3, 0.3, bad)[0] == -5
    assert o.temperature_update_gap(1.0, 0.3, 0.6, 10.0, tau_max=1.01)[1] == 1.01


def test_measured_gap_tracks_alpha_better_than_the_surrogate_off_model():
    # two-level rows whose gap is far from ln N + ln ln N = 14.4: scaling the entropy by
    # alpha through the measured gap lands closer to alpha than Eq. 4's surrogate does
    for delta in (10.0, 12.0):
        row = np.zeros((1, V_Q), np.float32)
        row[0, 9] = delta
        H0 = o.logprob_entropy(row, None, None, None, 1.0).entropy[0]
        gap = o.logit_gaps(row, None, 1.0)[0]
        for alpha in (0.9, 1.1):
            t_gap = o.temperature_update_gap(1.0, 1.0, alpha, gap)[1]
            t_eq4 = o.temperature_update(1.0, 1.0, alpha, V_Q)[1]
            r_gap = o.logprob_entropy(row, None, None, None, np.float32(t_gap)).entropy[0] / H0
            r_eq4 = o.logprob_entropy(row, None, None, None, np.float32(t_eq4)).entropy[0] / H0
            assert abs(r_gap - alpha) < abs(r_eq4 - alpha)
