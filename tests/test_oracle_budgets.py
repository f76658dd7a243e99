"""Pins for the oracle's difficulty ranking and Algorithm 1 (not gpu): hand-worked
batches, the algorithm's invariants (batch total constant, bounds respected, harder
questions never get less), and brute-force re-statements in plain Python."""
import math

import numpy as np
import pytest

from oracle import e3_oracle as o


def test_ranks_hand_worked():
    # average rewards: .75, .25, 1.0, .25, 0 (never sampled) -> descending: q2, q0, q1, q3, q4
    rc, k = o.difficulty_ranks([6, 2, 8, 1, 0], [8, 8, 8, 4, 0])
    assert rc == 0
    assert np.allclose(k, [2 / 5, 3 / 5, 1 / 5, 4 / 5, 5 / 5])
    # the question answered worst gets k = 1, the best k = 1/|D|
    rc, k = o.difficulty_ranks([0.0, 16.0], [16, 16])
    assert rc == 0 and list(k) == [1.0, 0.5]
    assert o.difficulty_ranks([1.0], [-1])[0] == -5


def test_ranks_are_a_permutation_over_D():
    rng = np.random.default_rng(0)
    n = 200
    cnt = rng.integers(1, 40, n)
    rew = rng.binomial(cnt, rng.uniform(0, 1, n)).astype(float)
    rc, k = o.difficulty_ranks(rew, cnt)
    assert rc == 0
    assert sorted(np.rint(k * n).astype(int)) == list(range(1, n + 1))
    avg = rew / cnt
    order = np.argsort(k)                      # rank 1 first
    assert all(avg[order[i]] >= avg[order[i + 1]] for i in range(n - 1))
    # plain-Python restatement: stable sort by descending average
    want = sorted(range(n), key=lambda i: (-avg[i], i))
    assert list(order) == want


def test_algorithm1_hand_worked():
    # B=4, G=8, bounds 4..12, k=(.25,.5,.75,1): start 4 each, 16 left, shares floor(16k/2.5)
    # = 1,3,4,6 -> 5,7,8,10 (30); 2 left go to the two hardest -> 5,7,9,11
    rc, g = o.allocate_budgets([0.25, 0.5, 0.75, 1.0], 8, 4, 12)
    assert rc == 0 and list(g) == [5, 7, 9, 11]
    # bounds equal to G (first pass over the data): nothing moves
    rc, g = o.allocate_budgets([0.1, 0.9, 0.5], 8, 8, 8)
    assert rc == 0 and list(g) == [8, 8, 8]
    # equal difficulty: equal budgets
    rc, g = o.allocate_budgets([0.5] * 6, 8, 4, 12)
    assert rc == 0 and list(g) == [8] * 6
    # cap binds: k=(0,0,1), G=8, 6..10: shares 0,0,6 -> 6,6,10 after cap (22 of 24);
    # the 2 left go, in descending k with ties by index, to q0 and q1 (q2 is full)
    rc, g = o.allocate_budgets([0.0, 0.0, 1.0], 8, 6, 10)
    assert rc == 0 and list(g) == [7, 7, 10]
    # Section 5.3's third pass: 64 questions, G=8, bounds 4..12
    k = (np.arange(64) + 1) / 64.0
    rc, g = o.allocate_budgets(k, 8, 4, 12)
    assert rc == 0 and g.sum() == 512 and g.min() >= 4 and g.max() <= 12
    assert all(a <= b for a, b in zip(g, g[1:]))


def _restate(k, G, G_min, G_max):
    B = len(k)
    total = B * G
    g = [G_min] * B
    rem = total - B * G_min
    s = 0.0
    for x in k:
        s += x
    for i in range(B):
        g[i] = min(G_max, g[i] + math.floor(rem * k[i] / s))
    left = total - sum(g)
    order = sorted(range(B), key=lambda i: (-k[i], i))
    while left > 0:
        for i in order:
            if left > 0 and g[i] < G_max:
                g[i] += 1
                left -= 1
    return g


def test_algorithm1_invariants_and_restatement():
    rng = np.random.default_rng(1)
    for trial in range(300):
        B = int(rng.integers(1, 80))
        G = int(rng.integers(1, 17))
        G_min = int(rng.integers(0, G + 1))
        G_max = int(rng.integers(G, G + 9))
        if trial % 3 == 0:
            k = (rng.permutation(B) + 1) / float(B)          # true normalised ranks
        else:
            k = rng.uniform(0, 1, B)
            k[rng.integers(0, B)] = 1.0
        rc, g = o.allocate_budgets(k, G, G_min, G_max)
        assert rc == 0
        assert g.sum() == B * G                              # batch total is constant
        assert g.min() >= G_min and g.max() <= G_max
        assert list(g) == _restate(list(k), G, G_min, G_max)
        order = np.argsort(k, kind="stable")
        gs = g[order]
        assert all(a <= b for a, b in zip(gs, gs[1:]))       # harder never gets less


def test_algorithm1_errors():
    assert o.allocate_budgets([0.5, 0.5], 8, 9, 12)[0] == -5   # G_min > G
    assert o.allocate_budgets([0.5, 0.5], 8, 4, 7)[0] == -5    # G_max < G
    assert o.allocate_budgets([0.0, 0.0], 8, 4, 12)[0] == -5   # no difficulty mass
    assert o.allocate_budgets([0.5, -0.1], 8, 4, 12)[0] == -5
    assert o.allocate_budgets([0.5, float("nan")], 8, 4, 12)[0] == -5
    assert o.allocate_budgets([], 8, 4, 12)[0] == 0


def test_bounds_curriculum():
    # Section 5.3: G = 8, +-2 per pass over the data, limits 4 and 12
    assert o.budget_bounds(8, 0, 2, 4, 12) == (0, 8, 8)
    assert o.budget_bounds(8, 1, 2, 4, 12) == (0, 6, 10)
    assert o.budget_bounds(8, 2, 2, 4, 12) == (0, 4, 12)
    assert o.budget_bounds(8, 5, 2, 4, 12) == (0, 4, 12)
    assert o.budget_bounds(8, 1, 2, 9, 12)[0] == -5
    assert o.budget_bounds(8, 1, 2, 4, 7)[0] == -5
