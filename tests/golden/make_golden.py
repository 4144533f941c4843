"""Writes the stored random-block tables under tests/golden/.  Calls only oracle/.

Run from the repository root:  python tests/golden/make_golden.py
Each file: a header line "H nb r seed g w global_mode", then H*nb rows of r integers.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import make_rand_idx  # noqa: E402

CASES = [
    # name, H, n, b, g, w, r, seed, global_mode
    ("rand_idx_cfg1_seed0", 2, 1024, 64, 2, 3, 3, 0, 0),
    ("rand_idx_cfg2_seed1", 12, 4096, 64, 2, 3, 3, 1, 0),
    ("rand_idx_cfg5_seed4_head0_3", 4, 16384, 64, 2, 3, 3, 4, 0),
    ("rand_idx_figure_seed7", 1, 12, 2, 1, 3, 1, 7, 0),
    ("rand_idx_leading_seed9", 3, 640, 64, 3, 5, 2, 9, 1),
]


def main():
    for name, H, n, b, g, w, r, seed, mode in CASES:
        t = make_rand_idx(H, n, b, g, w, r, seed, mode)
        with open(os.path.join(HERE, name + ".txt"), "w") as f:
            f.write(f"{H} {n // b} {r} {seed} {g} {w} {mode}\n")
            for row in t.reshape(-1, r):
                f.write(" ".join(str(int(x)) for x in row) + "\n")


if __name__ == "__main__":
    main()
