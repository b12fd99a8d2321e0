"""Writes tests/golden/perm_small.txt from the CPU oracle only.

Each line: seed b t N0 followed by the first entries of PERM(seed, b, t, N0) as
defined in oracle/perm.py.  The file is a regression anchor for the frozen
constants of that definition (the paper names no generator for Algorithm 1's
random partitions, so no published values exist).  Run: python tests/golden/make_golden.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import perm as P  # noqa: E402

CASES = [(0, 0, 1, 16), (0, 0, 2, 16), (0, 1, 1, 16), (1, 0, 1, 16), (0, 0, 0, 10),
         (0, 0, 1, 2000), (0, 49, 2, 100000), (123456789012, 7, 3, 1000000)]

if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "perm_small.txt")
    with open(out, "w") as fh:
        fh.write("# seed b t N0 perm[0:min(N0,24)] -- PERM as defined in oracle/perm.py (scalar form)\n")
        for seed, b, t, N0 in CASES:
            head = min(N0, 24)
            if N0 <= 4096:
                vals = P.perm_scalar(seed, b, t, N0)[:head]
            else:
                h, keys = P.half_width(N0), P.round_keys(seed, b, t)
                vals = []
                for j in range(head):
                    x = P.feistel_scalar(j, keys, h)
                    while x >= N0:
                        x = P.feistel_scalar(x, keys, h)
                    vals.append(x)
            fh.write(" ".join(str(v) for v in [seed, b, t, N0] + vals) + "\n")
    print("wrote", out)
