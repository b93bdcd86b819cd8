"""Writes tests/golden/oracle_tiny_item5.txt from the oracle alone (no GPU, no HIP library).

Usage: python tests/golden/make_golden.py
The paper prints no numeric example for the kernel, so this fixture is not a pin of the
oracle's correctness; it freezes the oracle's output on one work item of the Tiny workload
so that an accidental change to the oracle or to the input generators is noticed.
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2509_16518_amd import workloads as W  # noqa: E402

ITEM = 5


def compute():
    w = W.TINY
    q, k, v = W.make_qkv(w)
    indptr, indices = W.make_mask(w)
    out, lse = oracle.attention(q, k, v, w.M, w.N, w.scale, indptr, indices, items=np.array([ITEM]))
    return np.concatenate([out[0].reshape(-1), lse[0].reshape(-1)])


if __name__ == "__main__":
    vals = compute()
    with open(os.path.join(HERE, "oracle_tiny_item5.txt"), "w") as f:
        f.write("# oracle output for work item %d of workloads.TINY: out[16*64] then lse[16]; written by make_golden.py\n"
                % ITEM)
        for x in vals:
            f.write("%.17g\n" % x)
