"""Writes tests/golden/oracle_small.txt: outputs of the CPU oracle for two tiny seeded cases.

    python tests/golden/make_oracle_golden.py

Calls only `oracle/` and the seeded input generator.  The paper prints no worked numerical
example (so nothing here is the paper's), the file is a lock on the oracle's arithmetic: a
later change to the oracle that moves any of these numbers has to be deliberate.  The values
are printed with 17 significant digits (round-trip exact for fp64).
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import binattn_oracle as orc  # noqa: E402
from paper_2603_09582_amd import workloads as wl  # noqa: E402
from tests.helpers import bf16_bits  # noqa: E402

CASES = [("tiny_d8", 1, 1, 5, 8, 7), ("two_heads_d40", 1, 2, 7, 40, 8)]


def compute(B, H, N, d, seed):
    x = wl.make_inputs(wl.custom_workload(B, H, N, d, seed), device="cpu")
    res = orc.forward(bf16_bits(x.q), bf16_bits(x.k), bf16_bits(x.v), bf16_bits(x.bias), x.scale,
                      want=("O2", "O1"))
    return res


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small.txt")
    with open(out, "w") as f:
        f.write("# oracle outputs; written by tests/golden/make_oracle_golden.py (calls only oracle/)\n")
        f.write("# Eq. 5-7 and Alg. 1 as read in the oracle's header; inputs: workloads.custom_workload(B,H,N,d,seed) on the CPU\n")
        for name, B, H, N, d, seed in CASES:
            res = compute(B, H, N, d, seed)
            f.write(f"case {name} B={B} H={H} N={N} d={d} seed={seed}\n")
            for key in ("mu_q", "mu_k", "O2") + (("O1",) if N * d <= 64 else ()):
                a = np.asarray(res[key], dtype=np.float64).reshape(-1)
                f.write(f"{key} {a.size} " + " ".join(repr(float(v)) for v in a) + "\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
