"""Pins for the oracle's temperature scheduler, Eq. 4 and Eq. 5 (not gpu)."""
import math

import numpy as np
import pytest

from oracle import e3_oracle as o

V_Q = 151_936
D = math.log(V_Q) + math.log(math.log(V_Q))


def _next(tau, alpha, **kw):
    rc, nxt, tgt = o.temperature_update(tau, 1.0, alpha, V_Q, **kw)   # H_init/H_t = alpha
    assert rc == 0
    return nxt


def test_denominator_value():
    assert D == pytest.approx(14.4103727049, abs=1e-9)


def test_fixed_point_alpha_one():
    for tau in (0.3, 1.0, 1.7):
        rc, nxt, tgt = o.temperature_update(tau, 0.25, 0.25, V_Q)
        assert rc == 0 and nxt == tau and tgt == 0.25


def test_eq4_values():
    assert _next(1.0, 1.1) == pytest.approx(1 + math.log(1.1) / D, abs=1e-15)
    assert _next(1.0, 1.1) == pytest.approx(1.0066139982, abs=1e-9)
    assert _next(1.0, 0.9) == pytest.approx(0.9926885641, abs=1e-9)
    assert _next(1.0, 2.0) == pytest.approx(1.0481005727, abs=1e-9)
    assert _next(1.0, 0.5) == pytest.approx(0.9518994273, abs=1e-9)
    assert _next(1.2, 1.05) == pytest.approx(1.2 * (1 + 1.2 * math.log(1.05) / D), abs=1e-15)
    assert _next(1.2, 1.05) == pytest.approx(1.2048755045, abs=1e-9)
    assert _next(0.6, 1.25) == pytest.approx(0.6055745733, abs=1e-9)
    # alpha > 1 (entropy fell below target) raises tau, alpha < 1 lowers it; symmetric at tau = 1
    assert _next(1.0, 2.0) - 1 == pytest.approx(1 - _next(1.0, 0.5), abs=1e-15)


def test_eq5_schedule():
    # eta = 0.9, 480 steps, annealing from step 288 = floor(0.6 * 480) (Section 5.3 settings)
    H0, eta, ta, tm = 0.37, 0.9, 288, 480
    assert o.entropy_target(H0, 0, ta, tm, eta) == H0
    assert o.entropy_target(H0, 287, ta, tm, eta) == H0
    assert o.entropy_target(H0, 288, ta, tm, eta) == pytest.approx(H0, abs=1e-16)
    assert o.entropy_target(H0, 336, ta, tm, eta) == pytest.approx(0.9853553391 * H0, abs=1e-10)
    assert o.entropy_target(H0, 384, ta, tm, eta) == pytest.approx(0.95 * H0, abs=1e-15)
    assert o.entropy_target(H0, 480, ta, tm, eta) == pytest.approx(eta * H0, abs=1e-15)
    assert o.entropy_target(H0, 10_000, ta, tm, eta) == pytest.approx(eta * H0, abs=1e-15)
    assert o.entropy_target(H0, 5, -1, tm, eta) == H0                  # annealing off
    assert o.entropy_target(H0, 300, 288, 288, eta) == pytest.approx(eta * H0, abs=1e-15)
    vals = [o.entropy_target(H0, t, ta, tm, eta) for t in range(288, 481)]
    assert all(a >= b for a, b in zip(vals, vals[1:]))                 # monotone decay
    # the update uses the annealed target as the numerator of alpha
    rc, nxt, tgt = o.temperature_update(1.0, 0.30, H0, V_Q, t=384, t_anneal=ta, t_max=tm, eta=eta)
    assert rc == 0 and tgt == pytest.approx(0.95 * H0, abs=1e-15)
    assert nxt == pytest.approx(1 + math.log(0.95 * H0 / 0.30) / D, abs=1e-15)


def test_guards_and_clamps():
    for bad in (dict(tau_t=0.0), dict(tau_t=-1.0), dict(H_t=0.0), dict(H_init=0.0),
                dict(vocab=2), dict(tau_t=float("nan")), dict(H_t=float("inf"))):
        kw = dict(tau_t=1.0, H_t=0.2, H_init=0.2, vocab=V_Q)
        kw.update(bad)
        assert o.temperature_update(**kw)[0] == -5
    assert o.temperature_update(1.0, 0.2, 0.4, V_Q, tau_min=0.5, tau_max=1.01)[1] == 1.01
    assert o.temperature_update(1.0, 0.4, 0.2, V_Q, tau_min=0.99, tau_max=2.0)[1] == 0.99
    # factor <= 0 needs alpha < exp(-D/tau): error unless a positive floor is given
    assert o.temperature_update(1.0, 1.0, 1e-7, V_Q)[0] == -5
    assert o.temperature_update(1.0, 1.0, 1e-7, V_Q, tau_min=0.1)[1] == 0.1
    assert o.temperature_update(1.0, 0.2, 0.2, 3)[0] == 0


def _delta_entropy(N, tau, delta):
    w = (N - 1) * math.exp(-delta / tau)
    return math.log1p(w) + (delta / tau) * w / (1 + w)


def test_fig2_entropy_scales_roughly_linearly_with_alpha():
    # Section 4.2 / Fig. 2: applying Eq. 4 scales a small entropy by about alpha.
    # Checked on the Appendix-A two-level model with the oracle's own entropy.
    for delta in (15.0, 16.0):
        row = np.zeros((1, V_Q), np.float32)
        row[0, 5] = delta
        H0 = o.logprob_entropy(row, None, None, None, 1.0).entropy[0]
        assert H0 == pytest.approx(_delta_entropy(V_Q, 1.0, delta), abs=1e-10)
        for alpha in (0.8, 0.9, 1.1, 1.25):
            tau1 = _next(1.0, alpha)
            H1 = o.logprob_entropy(row, None, None, None, np.float32(tau1)).entropy[0]
            assert H1 / H0 == pytest.approx(alpha, rel=0.15)
    # and the exact-Delta relation tau1 = tau0 (1 + tau0 ln(alpha)/Delta) that Eq. 4
    # approximates stays within a few percent of it at Delta = ln N + ln ln N
    assert D == pytest.approx(math.log(V_Q) + math.log(math.log(V_Q)))
