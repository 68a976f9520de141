"""Writes the stored expected values under tests/golden/ by calling ONLY the
CPU oracle and the input generator (never the GPU library).

    python tests/golden/make_golden.py

c1_100iters.txt: the 256x256 single-tile workload (top edge 1.0, zero interior)
after 100 iterations: the residual norm and a handful of grid values as C99 hex
floats.  The paper (Sec. VI-C) prints no values for its Jacobi runs, so these are
oracle outputs, themselves pinned by tests/test_oracle_pins.py.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import jacobi_inputs as gen  # noqa: E402
import oracle  # noqa: E402

POINTS = [(1, 1), (1, 128), (2, 77), (10, 200), (50, 128), (100, 128), (100, 256), (101, 5)]


def main():
    w = gen.WORKLOADS["C1"]
    u, res = oracle.run(gen.generate(w), w.iters, w.residual_every)
    with open(os.path.join(HERE, "c1_100iters.txt"), "w") as f:
        f.write("# 256x256 fp64, top edge 1.0, others 0.0, interior 0.0, 100 Jacobi iterations\n")
        f.write("# written by tests/golden/make_golden.py from the CPU oracle\n")
        f.write(f"residual {res[0].hex()}\n")
        for (i, j) in POINTS:
            f.write(f"u {i} {j} {float(u[i, j]).hex()}\n")


if __name__ == "__main__":
    main()
