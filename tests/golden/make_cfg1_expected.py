#!/usr/bin/env python3
"""Writes tests/golden/cfg1_expected_samples.txt: the CPU oracle's result on the tiny
benchmark layer (N=1, Ci=3, 32x32 -> 16 channels, 3x3, stride 1, no padding; seed 1001) at
1200 output elements spread evenly over the output, for the test that drives the library from a
plain C program.  Calls only the oracle (Eq. 1, seven loops, fp64) and the seeded input generator.

    python tests/golden/make_cfg1_expected.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2306_14316_amd import workloads  # noqa: E402  (input generator only)


def main():
    L = workloads.layer(1)
    I, F = workloads.make_inputs(L)
    O, B = oracle.conv2d_direct(I.numpy(), F.numpy(), L.stride, L.pad)
    O, B = O.ravel(), B.ravel()
    idx = np.arange(0, O.size, 12)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_expected_samples.txt")
    with open(out, "w") as f:
        f.write("# CPU oracle on the tiny layer (1x3x32x32 -> 16, 3x3, s1, p0, seed 1001; Eq. 1 in fp64):\n")
        f.write("# flat NCHW output index, O (C99 hex double), sum|x||w| (C99 hex double).\n")
        f.write("# Written by tests/golden/make_cfg1_expected.py; %d of %d outputs.\n" % (idx.size, O.size))
        for i in idx:
            f.write("%d %s %s\n" % (i, float(O[i]).hex(), float(B[i]).hex()))
    print("wrote", out, idx.size, "samples")


if __name__ == "__main__":
    main()
