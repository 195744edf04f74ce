"""Writes the stored expected values under tests/golden/ by calling only oracle/.

Run from the repo root:  python tests/golden/make_golden.py
The paper prints no worked numeric example of the step, so the only stored
values are known-answer vectors of the stochastic-rounding hash (a reading of
Sec. 3.4, which leaves the random source open) as the oracle defines it; GPU
tests check the library's generator against the same file.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import numpy as np  # noqa: E402

from oracle import qgalore as Q  # noqa: E402

CASES = [
    (0, 1, 0), (0, 1, 1), (0, 1, 2), (0, 2, 0), (1, 1, 0), (0, 1, 255), (0, 1, 256), (0, 1, 262143),
    (0xDEADBEEF, 7, 12345), (0x0123456789ABCDEF, 100, 45088767), (2 ** 64 - 1, 2 ** 40 + 3, 2 ** 32 - 1),
    (42, 150000, 2 ** 32 + 5), (0, 0, 0),
]


def main():
    with open(os.path.join(HERE, "sr_hash_kat.txt"), "w") as f:
        f.write("# seed step idx -> hash32 (hex), per the SR generator defined in oracle/qgalore.py (reading of Sec. 3.4)\n")
        for seed, step, idx in CASES:
            h = int(Q.sr_hash(seed, step, np.array([idx], dtype=np.uint64))[0])
            f.write(f"{seed} {step} {idx} {h:08x}\n")


if __name__ == "__main__":
    main()
