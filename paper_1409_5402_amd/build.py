"""Compiles the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = [os.path.join(HERE, "csrc", "same_lda.hip")]
LIB = os.path.join(HERE, "libsame_lda.so")

# -ffp-contract=off: every binary32 step of the draw is rounded once (no fused multiply-add);
# packed-fp32 instructions are disabled for the device pass.
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fPIC", "-shared", "-Wall", "-Wextra", "-Wno-unused-value"]


STATS_LIB = os.path.join(HERE, "libsame_lda_stats.so")


def build(verbose: bool = False, stats: bool = False) -> str:
    """stats=True builds a second library whose draw kernel counts its own events (steps, trips, pmf terms,
    shared passes) into a device buffer given through same_lda_stats_buffer: for `bench.py --mode stats` only."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *(["-DSAME_STATS"] if stats else []), "-o", STATS_LIB if stats else LIB, *SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building the library")
    return STATS_LIB if stats else LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, stats="--stats" in sys.argv))
