"""Writes the frozen expected values under tests/golden/ that are not printed in the paper.
Calls only the CPU oracle.  Run from the repository root:  python tests/golden/make_golden.py"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def main():
    tours = oracle.init_tours(0xC0FFEE02, 16, 8)
    np.savetxt(os.path.join(HERE, "init_tours_seed_c0ffee02_n16.txt"), tours, fmt="%d",
               header="initial tours of restarts 0..7, seed 0xC0FFEE02, N=16 (self-pin: written by the oracle;\n"
                      "the paper only says the initial order is random, Section 1)")


if __name__ == "__main__":
    main()
