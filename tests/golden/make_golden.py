#!/usr/bin/env python3
"""Writes tests/golden/oracle_case_*.txt: outputs of the fp64 oracle on small seeded cases.

The paper prints no numeric worked example (all its numbers are in figures), so there is no
paper-valued fixture.  These files record what the oracle -- after it passed its pins (closed
forms, brute force, finite differences; see tests/test_oracle_*.py) -- returns on fixed inputs, so
that a later change to the oracle's arithmetic shows up as a diff against a stored value.  This
script calls only `oracle/` and the seeded input generators; nothing here comes from the GPU path.

    python tests/golden/make_golden.py          # rewrites the fixtures
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2501_06480_amd import synth  # noqa: E402

# name, N, L, heads, d, window side k (0 = no bias table), mask period, seed
CASES = [
    ("a_plain", 2, 5, 2, 4, 0, 0, 9001),
    ("b_bias_mask", 2, 9, 2, 4, 3, 2, 9002),
    ("c_ragged_blocks", 1, 16, 1, 32, 4, 0, 9003),
]


def inputs(case):
    name, N, L, heads, d, k, nW, seed = case
    C = heads * d
    q, kk, v, g = (synth.normal((N, L, C), seed * 16 + t).astype(np.float64) for t in range(4))
    bias = mask = None
    if k:
        bias = oracle.bias_gather(synth.bias_table(heads, k, seed, std=0.5), k)
    if nW:
        mask = np.where(synth.rng(seed + 7).random((nW, L, L)) < 0.25, -100.0, 0.0)
        mask[:, np.arange(L), np.arange(L)] = 0.0
    return q, kk, v, g, heads, float(d) ** -0.5, bias, mask


def compute(case):
    q, k, v, g, heads, scale, bias, mask = inputs(case)
    o = oracle.forward(q, k, v, heads, scale, bias, mask, threads=1)
    dq, dk, dv, db = oracle.backward(q, k, v, g, heads, scale, bias, mask, threads=1)
    return {"o": o, "dq": dq, "dk": dk, "dv": dv, "dbias": db}


def path(case):
    return os.path.join(HERE, f"oracle_case_{case[0]}.txt")


def main():
    for case in CASES:
        out = compute(case)
        with open(path(case), "w") as f:
            f.write(f"# fp64 oracle outputs, case {case[0]}: N={case[1]} L={case[2]} heads={case[3]} d={case[4]} "
                    f"k={case[5]} nW={case[6]} seed={case[7]}; written by tests/golden/make_golden.py\n")
            for name, a in out.items():
                f.write(f"{name} {' '.join(str(s) for s in a.shape)}\n")
                f.write(" ".join(float(x).hex() for x in a.ravel()) + "\n")
        print("wrote", path(case))


if __name__ == "__main__":
    main()
