"""Pins for the oracle's GRPO clipped objective, Eq. 1 (not gpu)."""
import math

import numpy as np
import pytest

from oracle import e3_oracle as o


def _one_token(r, A, eps=0.2):
    J, terms, means = o.grpo_objective([math.log(r)], [0.0], [0, 1], [A], [0, 1], eps)
    return terms[0]


def test_clip_cases_single_token():
    # A > 0: gains are capped at (1+eps) A;  A < 0: losses are not capped from above
    assert _one_token(1.5, 2.0) == pytest.approx(1.2 * 2.0, rel=1e-7)
    assert _one_token(0.5, 2.0) == pytest.approx(0.5 * 2.0, rel=1e-7)
    assert _one_token(1.5, -2.0) == pytest.approx(1.5 * -2.0, rel=1e-7)
    assert _one_token(0.5, -2.0) == pytest.approx(0.8 * -2.0, rel=1e-7)
    assert _one_token(1.1, 3.0) == pytest.approx(1.1 * 3.0, rel=1e-7)     # inside the clip range
    assert _one_token(1.0, -0.7) == pytest.approx(-0.7, rel=1e-7)
    assert _one_token(3.0, 1.0, eps=0.0) == pytest.approx(1.0)            # eps = 0: ratio pinned at 1


def test_hand_worked_batch():
    # 2 questions; q0 has rollouts of 2 and 1 tokens, q1 one rollout of 3 tokens
    lr = np.log(np.array([1.0, 1.5, 0.5, 1.0, 2.0, 0.9]))
    J, terms, means = o.grpo_objective(lr, np.zeros(6), [0, 2, 3, 6], [1.0, -1.0, 2.0], [0, 2, 3], 0.2)
    assert np.allclose(terms, [1.0, 1.2, -0.8, 2.0, 2.4, 1.8], rtol=1e-7)
    assert np.allclose(means, [1.1, -0.8, (2.0 + 2.4 + 1.8) / 3], rtol=1e-7)
    assert J == pytest.approx(((1.1 - 0.8) / 2 + 6.2 / 3) / 2, rel=1e-7)


def test_on_policy_value_is_mean_advantage():
    # r = 1 everywhere: J = mean_q mean_i A_i, which is 0 for group-normalised advantages
    rng = np.random.default_rng(0)
    sizes = [4, 8, 12, 6]
    goff = np.concatenate([[0], np.cumsum(sizes)])
    rewards = rng.integers(0, 2, goff[-1]).astype(np.float32)
    rewards[0:2] = [0, 1]; rewards[4:6] = [0, 1]; rewards[12:14] = [0, 1]; rewards[24:26] = [0, 1]
    adv = o.grpo_advantages(rewards, goff)
    lens = rng.integers(1, 50, goff[-1])
    soff = np.concatenate([[0], np.cumsum(lens)])
    lp = rng.normal(-2, 1, soff[-1]).astype(np.float32)
    J, _, means = o.grpo_objective(lp, lp, soff, adv, goff, 0.2)
    assert np.allclose(means, adv.astype(np.float32), atol=1e-12)
    assert J == pytest.approx(0.0, abs=1e-7)


def test_matches_numpy_restatement_and_edge_cases():
    rng = np.random.default_rng(1)
    sizes = [2, 0, 5, 3]
    goff = np.concatenate([[0], np.cumsum(sizes)])
    lens = np.array([3, 0, 7, 1, 4, 9, 2, 5, 6, 1])
    soff = np.concatenate([[0], np.cumsum(lens)])
    new = rng.normal(-2, 1, soff[-1]).astype(np.float32)
    old = (new + rng.normal(0, 0.3, soff[-1])).astype(np.float32)
    adv = rng.normal(0, 1, 10).astype(np.float32)
    eps = 0.2
    J, terms, means = o.grpo_objective(new, old, soff, adv, goff, eps)
    r = np.exp(new.astype(np.float64) - old.astype(np.float64))
    A_tok = np.repeat(adv.astype(np.float64), lens)
    want_terms = np.minimum(r * A_tok, np.clip(r, 1 - eps, 1 + eps) * A_tok)
    assert np.allclose(terms, want_terms, rtol=1e-14)
    want_means = np.array([want_terms[soff[i]:soff[i + 1]].mean() if lens[i] else 0.0 for i in range(10)])
    assert np.allclose(means, want_means, rtol=1e-14)
    want_J = np.mean([want_means[goff[q]:goff[q + 1]].mean() if sizes[q] else 0.0 for q in range(4)])
    assert J == pytest.approx(want_J, rel=1e-14)
    assert o.grpo_objective([], [], [0], [], [0], 0.2)[0] == 0.0
