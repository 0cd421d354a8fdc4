"""Writes tests/golden/projection_entries.txt from the oracle alone (no GPU code is imported):
entries of A for a few (seed, row, rank) triples, as hexadecimal fp64, so that an accidental
change to the oracle's generator (counter layout, bit-to-uniform map, Box-Muller pairing, scale)
shows up as a changed fixture.  The values are this build's definition of "N(0, 1/r) from a seed"
(the paper fixes only the distribution, Algorithm 1/2 sampling lines), not the paper's.
Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
import oracle  # noqa: E402

CASES = [(0, 0, 8), (1, 5, 16), (0x0123456789ABCDEF, 1000, 64), (2 ** 63 + 11, 2 ** 32 + 3, 256), (42, 16383, 32)]


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "projection_entries.txt")
    with open(out, "w") as f:
        f.write("# seed row r : A[row, 0..7] as hex fp64 (written by make_golden.py from oracle/ only)\n")
        for seed, row, r in CASES:
            vals = [oracle.A_elem(seed, row, k, r) for k in range(8)]
            f.write("%d %d %d : %s\n" % (seed, row, r, " ".join(float(v).hex() for v in vals)))
    print("wrote", out)


if __name__ == "__main__":
    main()
