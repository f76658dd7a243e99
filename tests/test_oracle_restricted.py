"""Pins for the oracle's top-k / top-p restricted sampler (CPU only).

The truncation rules are pinned against numpy's own selection routines and a plain
sort-and-cumsum nucleus on rows without repeated values, against hand-worked rows with
exact dyadic probabilities, and the draw itself against the truncated softmax by
chi-square over many seeds (with repeated values present, so that the choice inside a
level is covered too).
"""
import math

import numpy as np
import pytest
from scipy import stats

from oracle import e3_oracle as o


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns of values that bf16 represents exactly (upper half of binary32)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert (b & 0xFFFF == 0).all()
    return (b >> 16).astype(np.uint16)


def softmax(z, tau):
    a = z.astype(np.float64) / tau
    e = np.exp(a - a.max())
    return e / e.sum()


def test_no_truncation_reproduces_the_softmax():
    # k = 0 and p = 1 keep every column; logp is then the plain log-softmax
    rng = np.random.default_rng(0)
    z = rng.normal(0, 2, size=(1, 24)).astype(np.float32)
    n = 40_000
    res = o.sample_restricted(np.repeat(z, n, axis=0), None, 0.9, 0, 1.0, seed=5, nthreads=8)
    assert (res.kept == 24).all()
    p = softmax(z[0], np.float32(0.9))
    counts = np.bincount(res.token, minlength=24)
    chi2, pval = stats.chisquare(counts, p * n)
    assert pval > 1e-3, (chi2, pval)
    want = np.log(p)[res.token]
    assert np.abs(res.logp - want).max() < 1e-12


def test_top_k_matches_numpy_partition_and_keeps_ties():
    rng = np.random.default_rng(1)
    z = rng.normal(0, 3, size=(6, 500)).astype(np.float32)
    for k in (1, 2, 17, 499, 500, 1000):
        res = o.sample_restricted(z, None, 1.0, k, 1.0, seed=1)
        for r in range(6):
            kth = np.partition(z[r], -min(k, 500))[-min(k, 500)]
            assert res.kept[r] == int((z[r] >= kth).sum())
            assert z[r, res.token[r]] >= kth
    # repeated values at the cut are all kept
    row = np.array([[3, 1, 2, 2, 2, 0, 3, -1]], dtype=np.float32)
    assert o.sample_restricted(row, None, 1.0, 3, 1.0, seed=0).kept[0] == 5     # {3,3,2,2,2}
    assert o.sample_restricted(row, None, 1.0, 2, 1.0, seed=0).kept[0] == 2
    assert o.sample_restricted(row, None, 1.0, 1, 1.0, seed=0).kept[0] == 2     # both 3s


def test_top_k_one_is_the_argmax_with_logp_zero():
    rng = np.random.default_rng(2)
    z = rng.normal(0, 3, size=(50, 300)).astype(np.float32)
    res = o.sample_restricted(z, None, 0.7, 1, 1.0, seed=3)
    assert np.array_equal(res.token, z.argmax(axis=1))
    assert np.abs(res.logp).max() < 1e-15 and (res.kept == 1).all()


def test_top_p_matches_sort_and_cumsum_on_distinct_values():
    rng = np.random.default_rng(3)
    z = rng.normal(0, 2.5, size=(40, 400)).astype(np.float32)
    assert all(len(np.unique(z[r])) == 400 for r in range(40))
    for p in (0.05, 0.5, 0.9, 0.999):
        p32 = float(np.float32(p))
        res = o.sample_restricted(z, None, 1.3, 0, p, seed=7)
        for r in range(40):
            if res.near_cut[r]:
                continue
            pr = np.sort(softmax(z[r], np.float32(1.3)))[::-1]
            want = int(np.searchsorted(np.cumsum(pr), p32, side="left")) + 1   # smallest prefix >= p
            assert res.kept[r] == want, (p, r)
            srt = np.sort(z[r])[::-1]
            assert z[r, res.token[r]] >= srt[want - 1]


def test_hand_worked_dyadic_row():
    # logits 0..3 at tau = 1/ln2 give probabilities (1, 2, 4, 8)/15
    z = bf16_bits(np.array([[0.0, 1.0, 2.0, 3.0]], dtype=np.float32))
    tau = 1.0 / math.log(2.0)
    r = o.sample_restricted(z, None, tau, 0, 0.5, seed=0)       # 8/15 >= 0.5
    assert r.kept[0] == 1 and r.token[0] == 3 and abs(r.logp[0]) < 1e-6
    r = o.sample_restricted(z, None, tau, 0, 0.6, seed=0)       # 8/15 < 0.6 <= 12/15
    assert r.kept[0] == 2 and r.token[0] in (2, 3)
    want = math.log(8 / 12) if r.token[0] == 3 else math.log(4 / 12)
    assert abs(r.logp[0] - want) < 1e-6
    r = o.sample_restricted(z, None, tau, 0, 0.95, seed=0)      # 14/15 = 0.933 < 0.95
    assert r.kept[0] == 4
    # top-k first, then top-p on the renormalised top-k: k = 2 keeps {8, 4}/12, p = 0.7 > 8/12
    r = o.sample_restricted(z, None, tau, 2, 0.7, seed=0)
    assert r.kept[0] == 2
    r = o.sample_restricted(z, None, tau, 2, 0.6, seed=0)       # 8/12 = 0.667 >= 0.6
    assert r.kept[0] == 1
    # without the top-k step p = 0.6 keeps two levels (see above): the order matters


def test_draw_follows_the_truncated_softmax_with_repeated_values():
    # 12 columns, several repeated bf16 values; top-k = 7 cuts inside a repeated value
    vals = np.array([[2.0, 1.5, 2.0, 0.5, 1.5, 1.5, -1.0, 0.5, 0.0, -0.0, 3.0, -2.0]], dtype=np.float32)
    z = bf16_bits(vals)
    n = 60_000
    tau = np.float32(1.1)
    res = o.sample_restricted(np.repeat(z, n, axis=0), None, float(tau), 7, 0.97, seed=11, nthreads=8)
    # by hand: levels 3.0(1) 2.0(2) 1.5(3) 0.5(2) ...; top-k 7 -> C = 1,3,6,8 -> keep through 0.5 (8 columns)
    w = np.exp((vals[0].astype(np.float64) - 3.0) / tau)
    keep = vals[0] >= 0.5
    Mk = w[keep].sum()
    # top-p 0.97 of the top-k mass: cumulative by level
    lv = [(3.0, 1), (2.0, 2), (1.5, 3), (0.5, 2)]
    cum, kept_levels = 0.0, []
    for v, cnt in lv:
        cum += cnt * math.exp((v - 3.0) / tau)
        kept_levels.append(v)
        if cum >= float(np.float32(0.97)) * Mk:
            break
    keep2 = np.isin(vals[0], kept_levels)
    assert (res.kept == keep2.sum()).all()
    p = np.where(keep2, w, 0.0)
    p /= p.sum()
    counts = np.bincount(res.token, minlength=12)
    assert counts[~keep2].sum() == 0
    chi2, pval = stats.chisquare(counts[keep2], p[keep2] * n)
    assert pval > 1e-3, (chi2, pval)
    assert np.abs(res.logp - np.log(np.where(keep2, p, 1.0))[res.token]).max() < 1e-9


def _restate_draw(bits_row, tau, top_k, top_p, seed, row):
    """The library's definition of the restricted draw written again with numpy and the
    tests' own Philox: levels by bit pattern, race n_j w_j / E_j with the noise of stream 3
    indexed by the level's bit pattern, then the pos-th column with stream 4, index 0."""
    from tests import philox_np
    vals = (bits_row.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    key = np.where(bits_row & 0x8000, 0xFFFF - bits_row.astype(np.int64), bits_row.astype(np.int64) + 0x10000)
    patterns = sorted(set(bits_row.tolist()), key=lambda b: -int(key[np.flatnonzero(bits_row == b)[0]]))
    z1 = vals[np.flatnonzero(bits_row == patterns[0])[0]]
    n = np.array([(bits_row == b).sum() for b in patterns], dtype=np.float64)
    zl = np.array([vals[np.flatnonzero(bits_row == b)[0]] for b in patterns])
    w = np.exp((zl - z1) / tau)
    C, M = np.cumsum(n), np.cumsum(n * w)
    jk = len(patterns) - 1
    if 1 <= top_k < bits_row.size:
        jk = int(np.flatnonzero(C >= top_k)[0])
    jp = jk
    if top_p < 1.0:
        jp = int(np.flatnonzero(M[:jk + 1] >= top_p * M[jk])[0])
    words = philox_np.noise_words(seed, row, 3, np.array(patterns[:jp + 1], dtype=np.uint64))
    E = -np.log(((words >> np.uint32(9)).astype(np.float64) + 0.5) / 8388608.0)
    best = int(np.argmax(n[:jp + 1] * w[:jp + 1] / E))
    k23 = int(philox_np.noise_words(seed, row, 4, np.array([0]))[0]) >> 9
    pos = ((2 * k23 + 1) * int(n[best])) >> 24
    cols = np.flatnonzero(bits_row == patterns[best])
    return int(cols[pos]), int(C[jp]), (zl[best] - z1) / tau - math.log(M[jp])


@pytest.mark.parametrize("top_k,top_p", [(0, 1.0), (9, 1.0), (0, 0.8), (12, 0.9), (1, 0.5)])
def test_draw_matches_a_numpy_restatement(top_k, top_p):
    # few distinct values (many repeats), both signs, 300 rows with their own noise
    rng = np.random.default_rng(17)
    grid = np.array([-2.0, -1.0, -0.5, -0.0, 0.0, 0.25, 0.5, 1.0, 1.5, 2.0, 3.0], dtype=np.float32)
    rows, V, seed, base = 300, 40, 23, 1000
    z = bf16_bits(rng.choice(grid, size=(rows, V)))
    tau = np.float32(0.8)
    res = o.sample_restricted(z, None, float(tau), top_k, top_p, seed=seed, row_base=base, nthreads=4)
    for r in range(rows):
        if res.near_tie[r] or res.near_cut[r]:
            continue
        tok, kept, logp = _restate_draw(z[r], float(tau), top_k, float(np.float32(top_p)), seed, base + r)
        assert (res.token[r], res.kept[r]) == (tok, kept), r
        assert res.logp[r] == pytest.approx(logp, abs=1e-12)
    assert (res.near_tie | res.near_cut).mean() < 0.2


def test_all_equal_row_is_uniform_and_minus_zero_ranks_below_plus_zero():
    z = bf16_bits(np.full((1, 16), 0.25, dtype=np.float32))
    n = 32_000
    res = o.sample_restricted(np.repeat(z, n, axis=0), None, 1.0, 5, 0.3, seed=2, nthreads=8)
    assert (res.kept == 16).all()                     # one level: it cannot be cut
    chi2, pval = stats.chisquare(np.bincount(res.token, minlength=16))
    assert pval > 1e-3
    assert np.abs(res.logp - math.log(1 / 16)).max() < 1e-12
    zz = bf16_bits(np.array([[-0.0, 0.0, -0.0, -1.0]], dtype=np.float32))
    r = o.sample_restricted(zz, None, 1.0, 1, 1.0, seed=0)
    assert r.kept[0] == 1 and r.token[0] == 1         # +0 alone is the top level


def test_rows_are_keyed_by_global_row_id():
    rng = np.random.default_rng(5)
    z = rng.normal(0, 3, size=(8, 200)).astype(np.float32)
    a = o.sample_restricted(z, None, 1.0, 50, 0.9, seed=9, row_base=100)
    b = o.sample_restricted(z[3:5], None, 1.0, 50, 0.9, seed=9, row_base=103)
    assert np.array_equal(a.token[3:5], b.token) and np.array_equal(a.kept[3:5], b.kept)
