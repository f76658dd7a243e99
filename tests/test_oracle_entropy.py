"""Pins for the oracle's softmax statistics, entropy and log-prob (not gpu).

Everything here is a closed form, an invariant or a special case that reduces to a
library routine: Appendix A's softmax, the entropy definition, its decomposition,
and the exact form of the two-level Delta-model."""
import math

import numpy as np
import pytest
import torch
from scipy.special import log_softmax

from oracle import e3_oracle as o

V_Q = 151_936


def _H(row, tau=1.0):
    r = np.ascontiguousarray(row, dtype=np.float32).reshape(1, -1)
    return o.logprob_entropy(r, np.zeros(1, np.int32), None, None, tau).entropy[0]


def test_uniform_logits_give_ln_V_for_any_tau():
    for V in (1, 2, 7, 1024, V_Q):
        for tau in (0.3, 1.0, 2.0):
            assert _H(np.full(V, 1.75), tau) == pytest.approx(math.log(V), abs=1e-11)
    assert math.log(V_Q) == pytest.approx(11.931214658529, abs=1e-9)


def test_worked_distributions():
    z = np.log(np.array([1.0, 2.0, 3.0, 4.0]))
    # fp32-stored logits: compare against the entropy of the distribution they define
    zs = z.astype(np.float32).astype(np.float64)
    p = np.exp(zs) / np.exp(zs).sum()
    assert _H(z, 1.0) == pytest.approx(-(p * np.log(p)).sum(), abs=1e-13)
    # and, loosely, against the exact p = (.1,.2,.3,.4): H = 1.2798542258
    assert _H(z, 1.0) == pytest.approx(1.2798542258, abs=2e-7)
    # tau = 1/2 squares the weights: p ~ (1,4,9,16)/30
    q = np.array([1, 4, 9, 16]) / 30.0
    assert _H(z, 0.5) == pytest.approx(-(q * np.log(q)).sum(), abs=2e-7)
    assert -(q * np.log(q)).sum() == pytest.approx(1.0784767751, abs=1e-9)
    # p = (1/8,1/8,1/8,5/8): logits exactly representable -> tight
    z2 = np.array([0.0, 0.0, 0.0, math.log(5.0)])
    p2 = np.array([1, 1, 1, 5]) / 8.0
    assert _H(z2, 1.0) == pytest.approx(-(p2 * np.log(p2)).sum(), abs=2e-7)
    assert -(p2 * np.log(p2)).sum() == pytest.approx(1.0735428464, abs=1e-9)


def test_limits_in_tau():
    rng = np.random.default_rng(0)
    z = rng.normal(0, 2, 500)
    assert _H(z, 1e-3) == pytest.approx(0.0, abs=1e-9)      # tau -> 0+: one-hot
    assert _H(z, 1e6) == pytest.approx(math.log(500), abs=1e-9)  # tau -> inf: uniform
    hs = [_H(z, t) for t in (0.25, 0.5, 1.0, 2.0, 4.0)]
    assert all(a < b for a, b in zip(hs, hs[1:]))            # entropy grows with tau


def test_shift_and_scale_invariances():
    rng = np.random.default_rng(1)
    z = (rng.normal(0, 2, 300) * 64).round() / 64            # dyadic: shifts stay exact
    assert _H(z + 16.0, 0.7) == pytest.approx(_H(z, 0.7), abs=1e-12)
    # H(z, tau) = H(z/tau, 1) when z/tau is representable
    assert _H(z, 0.5) == pytest.approx(_H(z * 2.0, 1.0), abs=1e-12)
    assert _H(z, 2.0) == pytest.approx(_H(z * 0.5, 1.0), abs=1e-12)


def test_decomposition_equals_textbook_definition():
    rng = np.random.default_rng(2)
    for V, tau in ((5, 1.0), (64, 0.3), (1000, 1.4), (4096, 2.0)):
        z = rng.normal(0, 3, V).astype(np.float32)
        assert _H(z, tau) == pytest.approx(o.entropy_textbook(z, tau), rel=1e-12, abs=1e-13)


def _delta_model_exact(N, beta, delta):
    # Z = 1 + (N-1) e^{-beta delta};  H = ln Z + beta (N-1) delta e^{-beta delta} / Z
    w = (N - 1) * math.exp(-beta * delta)
    Z = 1.0 + w
    return math.log(Z) + beta * delta * w / Z


def test_delta_model_exact_form():
    # Appendix A's two-level model, without its small-entropy approximations.
    printed = {15.0: 0.7116256041, 16.0: 0.2859231621, 17.0: 0.1125321705}
    for delta, want in printed.items():
        row = np.zeros(V_Q, dtype=np.float32)
        row[12345] = delta
        assert _delta_model_exact(V_Q, 1.0, delta) == pytest.approx(want, abs=1e-9)
        assert _H(row, 1.0) == pytest.approx(want, abs=1e-9)
    row = np.zeros(1000, dtype=np.float32)
    row[3] = 6.0
    for tau in (0.5, 1.0, 1.5):
        assert _H(row, tau) == pytest.approx(_delta_model_exact(1000, 1 / tau, 6.0), abs=1e-12)
    # the approximation (N-1) beta delta e^{-beta delta} is close when entropy is small
    approx = (V_Q - 1) * 18.0 * math.exp(-18.0)
    row = np.zeros(V_Q, dtype=np.float32)
    row[0] = 18.0
    assert _H(row, 1.0) == pytest.approx(approx, rel=0.07)


def test_logprob_pins():
    rng = np.random.default_rng(3)
    z = rng.normal(0, 2, 50).astype(np.float32)
    for tau in (0.6, 1.0, 1.4):
        lp = o.log_softmax_row(z, tau)
        assert np.exp(lp).sum() == pytest.approx(1.0, abs=1e-13)
        t32 = float(np.float32(tau))                    # tau crosses the boundary as fp32
        assert np.allclose(lp, log_softmax(z.astype(np.float64) / t32), atol=1e-13, rtol=0)
    lp = o.log_softmax_row(np.full(V_Q, -3.0, np.float32), 0.9)
    assert np.allclose(lp, -math.log(V_Q), atol=1e-11)
    # gather through the training-side call
    rows = rng.normal(0, 2, (6, 40)).astype(np.float32)
    tgt = np.array([0, 39, 7, 7, 20, 1], np.int32)
    res = o.logprob_entropy(rows, tgt, None, None, 0.8)
    for r in range(6):
        assert res.logp[r] == pytest.approx(o.log_softmax_row(rows[r], 0.8)[tgt[r]], abs=1e-14)
    bad = o.logprob_entropy(rows, np.array([-1, 40, 0, 0, 0, 0], np.int32), None, None, 1.0)
    assert np.isnan(bad.logp[0]) and np.isnan(bad.logp[1]) and np.isfinite(bad.logp[2])


def test_bf16_rows_are_widened_exactly():
    t = torch.tensor([[0.0, 1.0, -2.5, 3.140625, 100.0, -0.0078125]], dtype=torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    f32 = t.float().numpy()
    a = o.logprob_entropy(bits, np.array([3], np.int32), None, None, 0.7)
    b = o.logprob_entropy(f32, np.array([3], np.int32), None, None, 0.7)
    assert a.entropy[0] == b.entropy[0] and a.logp[0] == b.logp[0]


def test_per_row_tau_and_stride():
    rng = np.random.default_rng(4)
    big = rng.normal(0, 2, (5, 48)).astype(np.float32)
    view = big[:, :40]                                      # row stride 48, V = 40
    taus = np.array([0.6, 0.8, 1.0, 1.2, 1.4], np.float32)
    res = o.logprob_entropy(view, np.zeros(5, np.int32), None, taus, 99.0)
    for r in range(5):
        assert res.entropy[r] == pytest.approx(_H(big[r, :40], float(taus[r])), abs=1e-14)


def test_batch_mean_entropy_and_mask():
    rng = np.random.default_rng(5)
    rows = rng.normal(0, 2, (9, 33)).astype(np.float32)
    mask = np.array([1, 0, 1, 1, 0, 0, 1, 1, 1], np.uint8)
    res = o.logprob_entropy(rows, np.zeros(9, np.int32), mask, None, 1.0)
    assert res.entropy_count == 6
    assert res.entropy_sum == pytest.approx(res.entropy[mask == 1].sum(), abs=1e-13)
    full = o.logprob_entropy(rows, np.zeros(9, np.int32), None, None, 1.0)
    assert full.entropy_count == 9
    assert full.entropy_mean == pytest.approx(full.entropy.mean(), abs=1e-13)
    uni = o.logprob_entropy(np.zeros((4, 1024), np.float32), None, None, None, 1.3)
    assert uni.entropy_mean == pytest.approx(math.log(1024), abs=1e-12)
    assert np.isnan(uni.logp).all()
