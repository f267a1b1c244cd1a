#!/usr/bin/env python3
"""Writes tests/golden/toy_suboptimality.txt: F(w_t) - F* after epochs 1, 2, 4, 8 of the synthetic
least-squares problem of tests/toy_problem.py for SGD, gradient quantisation (QSGD) and QESGD in
its push and server forms (the comparison of Sec. 5 on a problem that needs no dataset).  Every
number comes from the CPU oracle driven by tests/test_toy_qesgd.py::oracle_epochs; nothing here
touches the HIP library.  Run from the repository root:  python tests/golden/make_toy_suboptimality.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))                      # tests/
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))     # repository root

from oracle import qesgd_oracle as oracle  # noqa: E402
from test_toy_qesgd import TABLE_EPOCHS, suboptimality_table  # noqa: E402
from toy_problem import make_problem  # noqa: E402


def main():
    A, y, w_star = make_problem()
    table = suboptimality_table(oracle, A, y, w_star)
    out = os.path.join(HERE, "toy_suboptimality.txt")
    with open(out, "w") as fh:
        fh.write("# F(w_t) - F* after epochs " + ", ".join(str(e) for e in TABLE_EPOCHS) +
                 " (oracle, seed 3; written by make_toy_suboptimality.py)\n")
        for name, vals in table.items():
            fh.write(name + " " + " ".join(f"{v:.6e}" for v in vals) + "\n")
    print(open(out).read())


if __name__ == "__main__":
    main()
