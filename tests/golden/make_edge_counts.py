"""Writes tests/golden/edge_counts.txt from the CPU oracle only.

Run from the repo root:  python tests/golden/make_edge_counts.py
Columns: n k causal E.  The affiliated part n*log2(n) (Sec. 3.2.2: 2^l edges per
level-l span) is checked in closed form before writing.
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

GRAPHS = [(512, 4, 0), (8192, 8, 1), (65536, 4, 1)] + [(4096, k, 0) for k in (2, 4, 8, 16, 32)]


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "edge_counts.txt")
    with open(path, "w") as f:
        f.write("# n k causal E -- written by tests/golden/make_edge_counts.py (oracle only)\n")
        for n, k, causal in GRAPHS:
            deg = oracle.degrees(n, k, bool(causal))
            assert int(deg[n:].sum()) == n * int(np.log2(n))
            f.write("%d %d %d %d\n" % (n, k, causal, int(deg.sum())))


if __name__ == "__main__":
    main()
