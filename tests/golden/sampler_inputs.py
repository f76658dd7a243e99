"""Inputs of the stored-token regression (tests/golden/sampler_tokens.txt): a seeded
integer hash turned into bf16 logit patterns, so that the rows are the same bits on
every machine and numpy version.  Holds no arithmetic of the method; imports neither the
oracle nor the HIP binding (both are fed from here)."""
import numpy as np

# (label, rows, V, seed, row_base, tau): two widths that span several sampler tiles, an
# incomplete last super-tile (4096 columns) and an incomplete last chunk of 8
CASES = (
    ("narrow", 24, 1000, 11, 5, 1.0),
    ("ragged", 16, 9001, 12, 1 << 33, 0.7),
    ("wide", 8, 20_000, 13, 77, 1.3),
)


def _mix(x):
    """splitmix64 finaliser on uint64 arrays (wrapping arithmetic)."""
    x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return x ^ (x >> np.uint64(31))


def logits_bf16(rows, V, seed):
    """uint16 [rows, V] of bf16 bit patterns: values k / 16 with k a hash in [-128, 127]
    (|z| <= 8, at most 8 significant bits: exactly representable in bf16), plus +6 on one hashed column
    per row so that the rows are peaked like a policy's."""
    with np.errstate(over="ignore"):
        r = np.arange(rows, dtype=np.uint64)[:, None]
        c = np.arange(V, dtype=np.uint64)[None, :]
        h = _mix(r * np.uint64(0x9E3779B97F4A7C15) + c + np.uint64(seed) * np.uint64(0xD1342543DE82EF95))
        k = (h >> np.uint64(40)).astype(np.int64) % 256 - 128
        z = k.astype(np.float32) / 16.0
        peak = (_mix(r[:, 0] + np.uint64(seed)) % np.uint64(V)).astype(np.int64)
    z[np.arange(rows), peak] += 6.0
    bits = z.view(np.uint32)
    assert (bits & 0xFFFF == 0).all()           # exactly representable: no rounding involved
    return (bits >> 16).astype(np.uint16)
