"""Writes the stored expected values under tests/golden/ from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import pyr_oracle as orc  # noqa: E402


def pyramid_lengths():
    S, lens = 2048, [2048]
    for _ in range(32):
        S = orc.schedule_next(S, 64, 93, 100, 192)
        lens.append(S)
    path = os.path.join(HERE, "pyramid_lengths_2048_093_192.txt")
    with open(path, "w") as f:
        f.write(" ".join(str(x) for x in lens))
        f.write("\n# Length entering layers 0..31 and after layer 31 of the 64 x 2k pyramid workload:\n"
                "# S_{l+1} = max(half-up(0.93 * S_l), 192), window 64.  Algorithm 1 of the paper (decay of\n"
                "# the retention ratio, minimum PvC length); the ratio and the floor are this build's workload.\n"
                "# The test re-derives the chain with exact rational arithmetic.\n")


if __name__ == "__main__":
    pyramid_lengths()
