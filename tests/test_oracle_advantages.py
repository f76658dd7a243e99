"""Pins for the oracle's group-relative advantage, Eq. 2 (not gpu)."""
import math

import numpy as np
import pytest

from oracle import e3_oracle as o


def test_worked_group_1000():
    off = np.array([0, 4], np.int32)
    r = np.array([1, 0, 0, 0], np.float32)
    a0 = o.grpo_advantages(r, off, ddof=0)
    assert np.allclose(a0, [math.sqrt(3.0), -1 / math.sqrt(3.0), -1 / math.sqrt(3.0),
                            -1 / math.sqrt(3.0)], atol=1e-15)
    assert a0[0] == pytest.approx(1.7320508076, abs=1e-9)
    a1 = o.grpo_advantages(r, off, ddof=1)
    assert np.allclose(a1, [1.5, -0.5, -0.5, -0.5], atol=1e-15)


def test_binary_reward_closed_form():
    # k ones among n, population std: A(1) = sqrt((n-k)/k), A(0) = -sqrt(k/(n-k))
    for n, k in ((2, 1), (8, 3), (12, 11), (32, 1), (32, 31), (5, 2)):
        r = np.zeros(n, np.float32)
        r[:k] = 1
        np.random.default_rng(n * 100 + k).shuffle(r)
        a = o.grpo_advantages(r, np.array([0, n], np.int32))
        assert np.allclose(a[r == 1], math.sqrt((n - k) / k), atol=1e-14)
        assert np.allclose(a[r == 0], -math.sqrt(k / (n - k)), atol=1e-14)
    a = o.grpo_advantages(np.array([1] + [0] * 31, np.float32), np.array([0, 32], np.int32))
    assert a[0] == pytest.approx(5.5677643628, abs=1e-9)
    assert a[1] == pytest.approx(-0.1796053020, abs=1e-9)


def test_identical_rewards_give_zero():
    # Section 4.2: when all rollouts of a question have the same reward the advantage is zero.
    for val in (0.0, 1.0, 0.1, -3.7):
        for n in (1, 2, 7, 32):
            a = o.grpo_advantages(np.full(n, val, np.float32), np.array([0, n], np.int32),
                                  ddof=0, eps=1e-6)
            assert np.array_equal(a, np.zeros(n))
    a = o.grpo_advantages(np.array([0.3], np.float32), np.array([0, 1], np.int32), ddof=1)
    assert a[0] == 0.0


def test_moments_and_affine_invariance():
    rng = np.random.default_rng(11)
    sizes = [2, 3, 4, 8, 16, 32, 5]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    r = rng.normal(0, 1, off[-1]).astype(np.float32)
    for ddof in (0, 1):
        a = o.grpo_advantages(r, off, ddof=ddof)
        for g, n in enumerate(sizes):
            seg = a[off[g]:off[g + 1]]
            assert seg.sum() == pytest.approx(0.0, abs=1e-13)
            assert (seg ** 2).sum() == pytest.approx(n - ddof, rel=1e-13)
            ref = r[off[g]:off[g + 1]].astype(np.float64)
            assert np.allclose(seg, (ref - ref.mean()) / ref.std(ddof=ddof), atol=1e-13)
    # r -> 4 r + 2 (exact in fp32 for these dyadic values) leaves advantages unchanged
    rd = (rng.integers(-64, 64, off[-1]) / 16.0).astype(np.float32)
    a = o.grpo_advantages(rd, off)
    b = o.grpo_advantages(rd * 4 + 2, off)
    assert np.allclose(a, b, atol=1e-13)


def test_csr_edges():
    off = np.array([0, 0, 3, 3, 5], np.int32)           # empty groups in between
    r = np.array([1, 0, 1, 0, 1], np.float32)
    a = o.grpo_advantages(r, off)
    k = math.sqrt(0.5)
    assert np.allclose(a, [k, -2 * k, k, -1, 1], atol=1e-15)
    assert o.grpo_advantages(np.zeros(0, np.float32), np.array([0], np.int32)).size == 0
    # eps is added to sigma
    a = o.grpo_advantages(np.array([1, 0, 0, 0], np.float32), np.array([0, 4], np.int32),
                          eps=0.5)
    sig = math.sqrt(3) / 4
    assert a[0] == pytest.approx(0.75 / (sig + 0.5), abs=1e-15)
