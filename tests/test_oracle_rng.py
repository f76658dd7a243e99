"""Pins for the oracle's counter-based noise (not gpu).

The paper does not describe its sampler; the noise source is Philox4x32-10 as
published by Salmon et al. (SC'11).  It is pinned by the published known-answer
vectors and by a second implementation written for the tests."""
import os

import numpy as np

from oracle import e3_oracle as o
from tests import philox_np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            yield w[0:4], w[4:6], w[6:10]


def test_published_known_answers():
    n = 0
    for ctr, key, want in _kat_rows():
        got = o.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want
        n += 1
    assert n == 3


def test_second_implementation_agrees_word_for_word():
    rng = np.random.default_rng(7)
    ctr = rng.integers(0, 2**32, size=(2000, 4), dtype=np.uint64)
    key = rng.integers(0, 2**32, size=2, dtype=np.uint64)
    ref = philox_np.philox4x32_10(ctr[:, 0], ctr[:, 1], ctr[:, 2], ctr[:, 3], key[0], key[1])
    for j in range(0, 2000, 37):
        got = o.philox4x32_10(ctr[j].astype(np.uint32), key.astype(np.uint32))
        assert [int(got[i]) for i in range(4)] == [int(ref[i][j]) for i in range(4)]


def test_noise_addressing():
    # word(index) = philox(counter = (index/4, row lo, row hi, stream), key = seed)[index % 4]
    seed = 0x1234_5678_9ABC_DEF0
    row = (5 << 32) | 77
    for stream in (1, 2):
        for index in (0, 1, 2, 3, 4, 5, 1187, 151_935, 2**32 - 1):
            blk = o.philox4x32_10([index >> 2, row & 0xFFFFFFFF, row >> 32, stream],
                                  [seed & 0xFFFFFFFF, seed >> 32])
            assert o.noise_word(seed, row, stream, index) == int(blk[index & 3])
    idx = np.arange(0, 4096)
    ref = philox_np.noise_words(seed, row, 2, idx)
    got = np.array([o.noise_word(seed, row, 2, int(i)) for i in idx], dtype=np.uint32)
    assert np.array_equal(ref, got)


def test_uniform_is_strictly_inside_unit_interval_and_fp32_exact():
    assert o.uniform(0) == 2.0 ** -24
    assert o.uniform(0x1FF) == 2.0 ** -24           # low 9 bits are dropped
    assert o.uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert o.uniform(1 << 9) == 3 * 2.0 ** -24
    for w in (0, 511, 512, 0x80000000, 0xFFFFFFFF, 0x12345678):
        u = o.uniform(w)
        assert np.float32(u) == u                   # representable without rounding


def test_gumbel_range_and_definition():
    lo, hi = o.gumbel(0), o.gumbel(0xFFFFFFFF)
    assert abs(lo - (-np.log(-np.log(2.0 ** -24)))) < 1e-12
    assert abs(hi - (-np.log(-np.log1p(-(2.0 ** -24))))) < 1e-9
    assert -2.82 < lo < -2.80 and 16.6 < hi < 16.7
    w = np.array([1, 12345, 0x80000000, 0xDEADBEEF], dtype=np.uint32)
    ref = philox_np.gumbel_from_words(w)
    for i in range(4):
        assert abs(o.gumbel(int(w[i])) - ref[i]) < 1e-12


def test_bit_and_byte_frequencies():
    # sanity on 2^20 words of stream 1: each bit ~ 1/2, bytes ~ uniform
    idx = np.arange(1 << 20)
    w = philox_np.noise_words(42, 3, 1, idx)
    assert w[5] == o.noise_word(42, 3, 1, 5)
    bits = np.unpackbits(w.view(np.uint8)).mean()
    assert abs(bits - 0.5) < 5 * 0.5 / np.sqrt(32 * w.size)
    counts = np.bincount(w.view(np.uint8), minlength=256)
    exp = counts.sum() / 256
    chi2 = ((counts - exp) ** 2 / exp).sum()
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)
    # Gumbel moments: mean = Euler gamma, var = pi^2/6
    g = philox_np.gumbel_from_words(w)
    assert abs(g.mean() - 0.5772156649) < 5 * np.sqrt(np.pi ** 2 / 6 / w.size)
    assert abs(g.var() - np.pi ** 2 / 6) < 0.02


def test_streams_seeds_rows_differ():
    base = [o.noise_word(1, 0, 1, i) for i in range(64)]
    assert base != [o.noise_word(2, 0, 1, i) for i in range(64)]
    assert base != [o.noise_word(1, 1, 1, i) for i in range(64)]
    assert base != [o.noise_word(1, 0, 2, i) for i in range(64)]
    assert base == [o.noise_word(1, 0, 1, i) for i in range(64)]
