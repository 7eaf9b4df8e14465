"""Writes tests/golden/oracle_small_cases.txt from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_oracle_golden.py
The file is a regression fixture for the oracle's arithmetic (hex floats, so
every bit is kept).  It calls only ``oracle`` and the seeded input generator.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2203_08069_amd import inputs  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_cases.txt")


def compute_cases():
    cases = {}
    for name, dt in (("f32", np.float32), ("f64", np.float64)):
        A, B = inputs.tensor(0, 0, (4, 6), dt), inputs.tensor(0, 1, (6, 3), dt)
        cases[f"gemm_{name}"] = oracle.gemm(A, B).ravel()
        T = inputs.tensor(2, 0, (2, 3, 5), dt)
        c = inputs.tensor(2, 1, (5,), dt)
        T2 = inputs.tensor(2, 2, (2, 3, 5), dt)
        cases[f"ttv_{name}"] = oracle.ttv(T, c).ravel()
        cases[f"innerprod_{name}"] = np.array([oracle.innerprod(T, T2)])
        C = inputs.tensor(3, 1, (5, 2), dt)
        cases[f"ttm_{name}"] = oracle.ttm(T, C).ravel()
        Cf, Df = inputs.tensor(4, 1, (3, 2), dt), inputs.tensor(4, 2, (5, 2), dt)
        cases[f"mttkrp_{name}"] = oracle.mttkrp(T, Cf, Df).ravel()
        # the same two contractions along the other modes of the 2 x 3 x 5 tensor
        for mode in (0, 1):
            Cn = inputs.tensor(3, 1, (T.shape[mode], 2), dt)
            cases[f"ttm_mode{mode}_{name}"] = oracle.ttm_mode(mode, T, Cn).ravel()
        for mode in (1, 2):
            a, b = [m for m in (0, 1, 2) if m != mode]
            Ca, Db = inputs.tensor(4, 1, (T.shape[a], 2), dt), inputs.tensor(4, 2, (T.shape[b], 2), dt)
            cases[f"mttkrp_mode{mode}_{name}"] = oracle.mttkrp_mode(mode, T, Ca, Db).ravel()
    return cases


def main():
    with open(OUT, "w") as f:
        f.write("# written by tests/golden/make_oracle_golden.py from the CPU oracle only\n")
        f.write("# <case> <binary64 values as hex floats, row-major>\n")
        for name, vals in compute_cases().items():
            f.write(name + " " + " ".join(float(v).hex() for v in vals) + "\n")


if __name__ == "__main__":
    main()
