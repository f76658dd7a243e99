"""Pins for the oracle's two-level Gumbel-max sampler (not gpu).

The paper only says rollouts are sampled at a temperature; the procedure is the
library's.  It is pinned by (i) a from-scratch re-statement in numpy on tiny inputs,
including the two degenerate partitions that are the textbook flat Gumbel-max,
(ii) chi-square tests of sample frequencies against softmax(z/tau), and
(iii) determinism / addressing properties."""
import math

import numpy as np
import pytest
from scipy.stats import chisquare

from oracle import e3_oracle as o
from tests import philox_np
from tests.partition import LIB_PARTITION

NT = 8  # oracle threads for the frequency tests


def _restate(z, tau, seed, row, partition):
    """Two-level Gumbel-max written out again with numpy (independent of the C code)."""
    chunk, lanes, depth = partition
    V = z.size
    a = z.astype(np.float64) / float(np.float32(tau))
    cols = np.arange(V)
    tile = (cols // (chunk * lanes * depth)) * lanes + (cols % (chunk * lanes)) // chunk
    m = a.max()
    ntiles = -(-V // (chunk * lanes * depth)) * lanes
    mass = np.zeros(ntiles)
    np.add.at(mass, tile, np.exp(a - m))
    g_tile = philox_np.gumbel_from_words(philox_np.noise_words(seed, row, 1, np.arange(ntiles)))
    with np.errstate(divide="ignore"):
        score = np.where(mass > 0, m + np.log(mass) + g_tile, -np.inf)
    best = int(np.argmax(score))                      # first maximum = lowest index
    members = cols[tile == best]
    g_col = philox_np.gumbel_from_words(philox_np.noise_words(seed, row, 2, members))
    return int(members[int(np.argmax(a[members] + g_col))])


@pytest.mark.parametrize("partition", [(1, 1, 1), (64, 1, 1), (2, 3, 2), (8, 64, 16), (4, 2, 5)])
def test_matches_restatement_on_tiny_rows(partition):
    rng = np.random.default_rng(hash(partition) % 1000)
    for V in (1, 5, 40, 64, 333):
        z = rng.normal(0, 2, (12, V)).astype(np.float32)
        taus = rng.uniform(0.6, 1.4, 12).astype(np.float32)
        res = o.sample_entropy(z, taus, 1.0, seed=99, row_base=1000, partition=partition)
        for r in range(12):
            if res.near_tie[r]:
                continue
            assert res.token[r] == _restate(z[r], taus[r], 99, 1000 + r, partition)


def test_library_partition_shape():
    chunk, lanes, depth = LIB_PARTITION
    assert (chunk, lanes, depth) == (8, 64, 8)
    nt = lambda V: o.num_tiles(V, LIB_PARTITION)
    tile_of = lambda c: o.tile_of(c, LIB_PARTITION)
    assert nt(151_936) == 38 * 64 and nt(1024) == 64 and nt(4096) == 64
    assert nt(4097) == 128
    # columns 0..7 -> tile 0, 8..15 -> tile 1, ..., 504..511 -> tile 63, 512.. wraps to tile 0
    assert [tile_of(c) for c in (0, 7, 8, 511, 512, 519, 4095, 4096, 4104)] == \
        [0, 0, 1, 63, 0, 0, 63, 64, 65]
    sizes = np.bincount([tile_of(c) for c in range(4096 + 100)], minlength=128)
    assert (sizes[:64] == 64).all() and sizes[64:76].tolist() == [8] * 12 and sizes[76] == 4


def _freq_test(z, tau, partition, draws, seed):
    V = z.size
    rows = np.broadcast_to(z.astype(np.float32), (draws, V))    # same row, different noise rows
    res = o.sample_entropy(rows, None, tau, seed=seed, row_base=0, partition=partition,
                           nthreads=NT)
    p = np.exp(o.log_softmax_row(z.astype(np.float32), tau))
    counts = np.bincount(res.token, minlength=V).astype(np.float64)
    expect = p * draws
    small = expect < 5.0                                         # pool sparse bins
    if small.sum() > 1:
        counts = np.append(counts[~small], counts[small].sum())
        expect = np.append(expect[~small], expect[small].sum())
    stat, pval = chisquare(counts, expect)
    return pval


def test_frequencies_follow_softmax_flat_and_tiled():
    rng = np.random.default_rng(5)
    draws = 1_000_000
    z8 = np.array([0.0, 1.0, 2.0, 3.0, -1.0, 0.5, 2.5, 1.5])
    for partition in ((1, 1, 1), (8, 1, 1), (2, 2, 1), (1, 2, 2)):
        assert _freq_test(z8, 1.0, partition, draws, seed=11) > 1e-4
    z64 = rng.normal(0, 2, 64)
    for partition, tau in (((1, 1, 1), 0.7), ((64, 1, 1), 1.3), ((4, 4, 2), 1.0), ((8, 64, 16), 0.6)):
        assert _freq_test(z64, tau, partition, draws, seed=12) > 1e-4


def test_frequencies_library_partition_V1024():
    rng = np.random.default_rng(6)
    z = rng.normal(0, 2, 1024)
    z[[3, 500, 1000]] += 5.0
    assert _freq_test(z, 1.0, LIB_PARTITION, 200_000, seed=13) > 1e-4
    assert _freq_test(z, 1.0, (1024, 1, 1), 200_000, seed=13) > 1e-4     # flat, same target law


def test_a_wrong_sampler_would_fail_the_frequency_test():
    # sanity of the test itself: tau mismatched by 10% is rejected at this sample size
    z8 = np.array([0.0, 1.0, 2.0, 3.0, -1.0, 0.5, 2.5, 1.5])
    rows = np.broadcast_to(z8.astype(np.float32), (1_000_000, 8))
    res = o.sample_entropy(rows, None, 1.1, seed=11, partition=(1, 1, 1), nthreads=NT)
    p = np.exp(o.log_softmax_row(z8.astype(np.float32), 1.0))
    counts = np.bincount(res.token, minlength=8)
    assert chisquare(counts, p * 1_000_000)[1] < 1e-6


def test_determinism_and_row_base():
    rng = np.random.default_rng(8)
    z = rng.normal(0, 2, (16, 700)).astype(np.float32)
    a = o.sample_entropy(z, None, 1.0, seed=5, row_base=100, partition=LIB_PARTITION)
    b = o.sample_entropy(z, None, 1.0, seed=5, row_base=100, partition=LIB_PARTITION, nthreads=4)
    assert np.array_equal(a.token, b.token) and np.array_equal(a.logp, b.logp)
    # rows 8..15 sampled on their own with row_base moved = same tokens
    c = o.sample_entropy(z[8:], None, 1.0, seed=5, row_base=108, partition=LIB_PARTITION)
    assert np.array_equal(a.token[8:], c.token)
    d = o.sample_entropy(z, None, 1.0, seed=6, row_base=100, partition=LIB_PARTITION)
    assert not np.array_equal(a.token, d.token)
    # logp and entropy agree with the training-side call on the sampled tokens
    t = o.logprob_entropy(z, a.token, None, None, 1.0)
    assert np.array_equal(t.logp, a.logp) and np.array_equal(t.entropy, a.entropy)


def _first_noise_collision(stream, seed, row, n):
    """Two indices i < j < n whose noise words give the same 23-bit uniform (a birthday
    collision: about n^2 / 2^24 of them are expected)."""
    seen = {}
    for idx in range(n):
        k = o.noise_word(seed, row, stream, idx) >> 9
        if k in seen:
            return seen[k], idx
        seen[k] = idx
    return None


@pytest.mark.parametrize("level", [1, 2])
def test_exact_ties_go_to_the_lowest_index_and_are_flagged(level):
    # an exact tie needs equal logits AND equal noise: take two columns whose uniforms
    # collide, give them the same logit and push every other column far below
    n, seed, row = 12_000, 5, 77
    pair = _first_noise_collision(level, seed, row, n)
    assert pair is not None
    i, j = pair
    z = np.full((1, n), -300.0, np.float32)
    z[0, i] = z[0, j] = 1.25
    # level 1: every column its own tile (tile noise indexed by the column);
    # level 2: one tile holding the whole row (column noise decides)
    partition = (1, 1, 1) if level == 1 else (n, 1, 1)
    res = o.sample_entropy(z, None, 1.0, seed=seed, row_base=row, partition=partition)
    assert res.token[0] == i                       # the lower of the two
    assert res.near_tie[0] == 1
    top = res.diag[0, 0:2] if level == 1 else res.diag[0, 2:4]
    assert top[0] == top[1]


def test_equal_masses_and_single_column_rows():
    # two tiles, identical mass: decided by the noise, not flagged unless scores are close
    z = np.zeros((1, 4), np.float32)
    res = o.sample_entropy(z, None, 1.0, seed=1, partition=(2, 2, 1))
    assert 0 <= res.token[0] < 4
    # degenerate one-column row
    one = o.sample_entropy(np.array([[3.5]], np.float32), None, 0.5, seed=1, partition=LIB_PARTITION)
    assert one.token[0] == 0 and one.logp[0] == 0.0 and one.entropy[0] == 0.0
    assert one.near_tie[0] == 0 and one.diag[0, 1] == -math.inf and one.diag[0, 3] == -math.inf


def test_near_tie_flag_rule():
    # diag holds the top-two scores per level; the flag is their relative closeness at 1e-5
    rng = np.random.default_rng(9)
    z = rng.normal(0, 2, (4000, 24)).astype(np.float32)
    res = o.sample_entropy(z, None, 1.0, seed=3, partition=(4, 3, 2), nthreads=NT)
    s1, s2, c1, c2 = res.diag.T
    assert (s1 >= s2).all() and (c1 >= c2).all()
    def close(x, y):
        return (x - y) <= 1e-5 * np.maximum(np.maximum(np.abs(x), np.abs(y)), 1.0)
    want = close(s1, s2) | close(c1, c2)
    assert np.array_equal(want.astype(np.uint8), res.near_tie)
    assert res.near_tie.mean() < 0.01
    # the margin itself: among very many tiny rows some have a top-two gap between 1e-7 and
    # 1e-5 (relative); exactly those and the closer ones are flagged
    z = rng.normal(0, 2, (600_000, 8)).astype(np.float32)
    res = o.sample_entropy(z, None, 1.0, seed=4, partition=(4, 1, 1), nthreads=NT)
    s1, s2, c1, c2 = res.diag.T
    def rel_gap(x, y):
        return (x - y) / np.maximum(np.maximum(np.abs(x), np.abs(y)), 1.0)
    gap = np.minimum(rel_gap(s1, s2), rel_gap(c1, c2))
    assert np.array_equal((gap <= 1e-5).astype(np.uint8), res.near_tie)
    assert ((gap > 1e-7) & (gap <= 1e-5)).sum() >= 3
    assert ((gap > 1e-5) & (gap <= 1e-4)).sum() >= 3          # and just outside: not flagged
