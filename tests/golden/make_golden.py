"""Writes tests/golden/c1_oracle_samples.txt: sampled outputs of the fp64
definition oracle on configuration c1 (seed 0).  Calls only oracle/ and the
input generator; the values guard against accidental changes of either."""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import bb_inputs                      # noqa: E402
from oracle import oracle as orc      # noqa: E402


def main():
    X, g, W1, W3, W2 = (bb_inputs.bits(t) for t in bb_inputs.make_config("c1"))
    rows = [0, 17, 63]
    cols = [0, 1, 100, 255]
    Y = orc.rmsnorm_swiglu_ffn(X, g, W1, W3, W2, 1e-6, rows=rows)
    with open(os.path.join(HERE, "c1_oracle_samples.txt"), "w") as fh:
        fh.write("# row col value(hex float64): oracle output on config c1, seed 0\n")
        for k, r in enumerate(rows):
            for c in cols:
                fh.write(f"{r} {c} {float(Y[k, c]).hex()}\n")


if __name__ == "__main__":
    main()
