"""Writes tests/golden/sampler_golden.txt from the CPU oracle alone.

The generator's constants are this repository's specification (the paper gives
no generator), so these vectors freeze that specification; the test suite also
checks them against a second, differently written implementation.
Run:  python tests/golden/make_sampler_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402

CASES = [
    # B P H  W  k mode per_sample seed stream
    (2, 0, 4, 4, 2, 0, 1, 0, 0),
    (1, 1, 6, 6, 1, 0, 1, 1, 1001),
    (2, 1, 4, 6, 3, 0, 1, 2, 2002),
    (2, 0, 5, 7, 2, 0, 1, 3, 3),
    (2, 0, 4, 4, 2, 1, 1, 0, 0),
    (2, 0, 4, 4, 2, 0, 0, 0, 0),
    (1, 0, 14, 14, 2, 0, 1, 0, 0),
    (1, 0, 3, 3, 3, 0, 1, 18446744073709551615, 18446744073709551615),
]


CELL_CASES = [
    # B P H  W  k cell mode per_sample seed stream
    (2, 0, 6, 6, 4, 3, 0, 1, 0, 0),
    (1, 1, 7, 10, 5, 3, 0, 1, 7, 70),
    (2, 0, 8, 8, 4, 4, 0, 1, 1, 2),
    (1, 1, 14, 14, 8, 4, 0, 1, 3, 4),
    (2, 0, 9, 9, 3, 3, 1, 1, 5, 6),
    (2, 1, 5, 11, 2, 4, 0, 0, 18446744073709551615, 9),
]


def write_cells():
    path = os.path.join(HERE, "sampler_cells_golden.txt")
    with open(path, "w") as f:
        f.write("# keep-index vectors of the 3 x 3 and 4 x 4 cell samplers, written by tests/golden/make_sampler_golden.py\n")
        f.write("# from the CPU oracle.  Not from the paper: they freeze this repository's sampler specification.\n")
        f.write("# Format:  B P H W k cell mode per_sample seed stream : idx...\n")
        for c in CELL_CASES:
            B, P, H, W, k, cell, mode, ps, seed, stream = c
            idx = oracle.sample_indices_cells(B, P, H, W, k, cell, seed, stream, mode=mode, per_sample=bool(ps))
            f.write(" ".join(str(v) for v in c) + " : " + " ".join(str(int(v)) for v in idx) + "\n")
    print("wrote", path)


def main():
    write_cells()
    path = os.path.join(HERE, "sampler_golden.txt")
    with open(path, "w") as f:
        f.write("# keep-index vectors written by tests/golden/make_sampler_golden.py from the CPU oracle.\n")
        f.write("# Not from the paper (it defines no generator): they freeze this repository's sampler\n")
        f.write("# specification.  Format:  B P H W k mode per_sample seed stream : idx...\n")
        for c in CASES:
            B, P, H, W, k, mode, ps, seed, stream = c
            idx = oracle.sample_indices(B, P, H, W, k, seed, stream, mode=mode, per_sample=bool(ps))
            f.write(" ".join(str(v) for v in c) + " : " + " ".join(str(int(v)) for v in idx) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
