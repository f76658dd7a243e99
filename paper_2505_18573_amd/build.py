"""Build libe3.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libe3.so")
SOURCES = ["e3_api.hip", "vocab_pass.hip", "restricted.hip", "restricted_select.hip", "probe.hip", "advantages.hip", "objective.hip",
           "scheduler.cpp", "budget.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fno-gpu-rdc", "-ffp-contract=on",
    # packed fp32 VALU forms are not used
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra=()) -> str:
    cmd = [HIPCC, *FLAGS, *extra, "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    # hipcc's host pass does not know the device-only target feature and says so once
    # per function; drop that line, keep everything else
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if err.strip():
        print(err)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed with status {res.returncode}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
