"""A second, vectorised Philox4x32-10 written for the tests only (numpy, uint64
products), used to pin the oracle's scalar C one word for word.  Follows Salmon et
al., SC'11, Section 3.3: ten rounds of two 32x32->64 multiplies with the key bumped
by the two Weyl constants between rounds."""
import numpy as np

_MUL = (np.uint64(0xD2511F53), np.uint64(0xCD9E8D57))
_WEYL = (0x9E3779B9, 0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    c = [np.asarray(x, dtype=np.uint64) & _MASK for x in (c0, c1, c2, c3)]
    c = list(np.broadcast_arrays(*c))
    k = [int(k0) & 0xFFFFFFFF, int(k1) & 0xFFFFFFFF]
    for rnd in range(10):
        if rnd:
            k = [(k[0] + _WEYL[0]) & 0xFFFFFFFF, (k[1] + _WEYL[1]) & 0xFFFFFFFF]
        left = _MUL[0] * c[0]
        right = _MUL[1] * c[2]
        c = [(right >> np.uint64(32)) ^ c[1] ^ np.uint64(k[0]), right & _MASK,
             (left >> np.uint64(32)) ^ c[3] ^ np.uint64(k[1]), left & _MASK]
    return [x.astype(np.uint32) for x in c]


def noise_words(seed, row, stream, indices):
    """Words of the library's noise addressing for an array of indices."""
    idx = np.asarray(indices, dtype=np.uint64)
    out = philox4x32_10(idx >> np.uint64(2), row & 0xFFFFFFFF, (row >> 32) & 0xFFFFFFFF, stream,
                        seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    sel = (idx & np.uint64(3)).astype(np.int64)
    stacked = np.stack(out, axis=0)
    return stacked[sel, np.arange(idx.size)]


def gumbel_from_words(words):
    k = (np.asarray(words, dtype=np.uint32) >> np.uint32(9)).astype(np.float64)
    u = (k + 0.5) / 8388608.0
    return -np.log(-np.log(u))
