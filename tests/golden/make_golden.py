"""Writes tests/golden/mixing_tables.txt from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
The file freezes the neighbour tables of the seeded randomized ring (Sec. 3, Eq. 8; the
shared-seed rule of Sec. 4) for a few (n, seed, step), so that a later change to either
the oracle or the library that moves a single index shows up as a diff.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import psgd_oracle as orc  # noqa: E402

CASES = [(1, 0, 0), (2, 0, 0), (3, 7, 1), (5, 3001, 0), (8, 3001, 9), (16, 3002, 0),
         (16, 3002, 49), (64, 3003, 0), (64, 3005, 19), (128, 3004, 99),
         (64, 2 ** 64 - 1, 2 ** 40)]


def main():
    out = ["# n seed step : sigma(0..n-1) | nbr rows (self left right) flattened",
           "# written by tests/golden/make_golden.py from oracle/psgd_oracle.py only"]
    for n, seed, step in CASES:
        sigma = orc.permutation(n, seed, step)
        nbr, _ = orc.neighbour_table(orc.TOPO_RAND_RING, n, seed, step)
        out.append("%d %d %d : %s | %s" % (n, seed, step, " ".join(map(str, sigma)),
                                           " ".join(str(int(v)) for v in nbr.reshape(-1))))
    with open(os.path.join(HERE, "mixing_tables.txt"), "w") as f:
        f.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main()
