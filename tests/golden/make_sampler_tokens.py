#!/usr/bin/env python3
"""Writes tests/golden/sampler_tokens.txt: the tokens the oracle draws, with the column
partition (8, 64, 8) that include/e3.h freezes, for the rows of sampler_inputs.py.

The file pins the token stream of (seed, row, logits): a later change of the partition, of
the noise addressing or of the tie rule, on either side, shows up as a difference against
stored values rather than as two sides that moved together.  Calls only oracle/ (and the
input generator); run from the repository root:  python tests/golden/make_sampler_tokens.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import e3_oracle as o                     # noqa: E402
from tests.golden import sampler_inputs as si         # noqa: E402

PARTITION = (8, 64, 8)      # written out here on purpose: the stored tokens belong to this partition
SAMPLER_SEED = 2025


def main():
    out = os.path.join(HERE, "sampler_tokens.txt")
    with open(out, "w") as f:
        f.write("# tokens of the two-level Gumbel-max sampler (include/e3.h: e3_sample_entropy),\n"
                "# column partition (chunk, lanes, depth) = (8, 64, 8), sampler seed 2025,\n"
                "# inputs: tests/golden/sampler_inputs.py; written by make_sampler_tokens.py from\n"
                "# the CPU oracle alone.  The paper (Section 5.1) samples at a temperature without\n"
                "# describing a sampler: these values pin the library's definition, not the paper.\n"
                "# line: label row token near_tie\n")
        for label, rows, V, seed, row_base, tau in si.CASES:
            bits = si.logits_bf16(rows, V, seed)
            res = o.sample_entropy(bits, None, tau, SAMPLER_SEED, row_base, partition=PARTITION)
            for r in range(rows):
                f.write(f"{label} {r} {int(res.token[r])} {int(res.near_tie[r])}\n")
    print(out)


if __name__ == "__main__":
    main()
