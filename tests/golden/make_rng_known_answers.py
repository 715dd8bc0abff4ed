#!/usr/bin/env python3
"""Writes tests/golden/rng_known_answers.txt: frozen outputs of the oracle's counter-based draw.

Calls only ``oracle/``.  The file freezes the function: an edit that changes the draw (a constant, a
shift, the order of the steps, the key derivation) no longer reproduces these lines, whichever
sides of the build the edit was applied to.  Run from the repository root:
    python tests/golden/make_rng_known_answers.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import rng  # noqa: E402

CASES = [
    (0, 0, 0), (0, 0, 1), (0, 0, 2), (1, 0, 0), (0, 1, 0), (1, 1, 1),
    (4, 7, 12345), (5, 0, 0xFFFFFFFF), (5, 0, 0x100000000), (5, 0, 0x100000001),
    (2 ** 63 + 5, 77, 123456789), (3, 4, (1 << 40) + 17), (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFFFFFFFFFF),
    (20240911, 31, 167772160 * 4 + 3),
]


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "rng_known_answers.txt")
    with open(out, "w") as f:
        f.write("# Frozen outputs of oracle/rng.py (written by make_rng_known_answers.py, which calls only oracle/).\n")
        f.write("# format: seed offset gid | k0 k1 | draw_u32 | uniform24 numerator (u = numerator * 2^-24)\n")
        for seed, offset, gid in CASES:
            k0, k1 = rng.derive_key(seed, offset)
            x = int(rng.draw_u32(k0, k1, np.array([gid], dtype=np.uint64))[0])
            u = float(rng.uniform24(seed, offset, np.array([gid], dtype=np.uint64))[0])
            f.write("%d %d %d | 0x%08X 0x%08X | 0x%08X | %d\n" % (seed, offset, gid, k0, k1, x, int(u * 2 ** 24)))
    print("wrote", out)


if __name__ == "__main__":
    main()
