"""Writes the stored expected values under tests/golden/ from the CPU oracle.

Calls only ``oracle/`` and the seeded input generator; never the GPU path.
Run from the repository root:  python tests/golden/make_golden.py

c1_tiny_y.txt: the oracle's fp64 output for the tiny configuration
(M=1, d_model=512, d_ff=1536, bf16 inputs, seed 0), one C99 hex float per
line, so that a later change to the oracle or the generator cannot go
unnoticed.  The paper prints no worked numerical example for this block, so
no fixture here carries a value from the paper.
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import dfk_inputs as di          # noqa: E402
from oracle import oracle        # noqa: E402


def main():
    t = di.mlp_inputs(1, 512, 1536, seed=0, dtype="bf16")
    Y = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_tiny_y.txt")
    with open(out, "w") as f:
        f.write("# oracle fp64 Y, M=1 d_model=512 d_ff=1536 bf16 seed=0; written by make_golden.py\n")
        for v in Y[0]:
            f.write(float(v).hex() + "\n")
    print("wrote", out, len(Y[0]), "values")


if __name__ == "__main__":
    main()
