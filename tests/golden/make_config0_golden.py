#!/usr/bin/env python3
"""Writes tests/golden/config0_oracle.txt: what the CPU oracle computes for benchmark
configuration 0 (seed 20251106).  Calls only the oracle and the input generator -- never the GPU
library -- so the stored values can serve as expected values for both.

    python tests/golden/make_config0_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle
from moska_inputs import config, generate


def main():
    inp = generate(config(0), seed=20251106)
    st = oracle.decode_step(inp)
    p = inp.prob
    with open(os.path.join(HERE, "config0_oracle.txt"), "w") as f:
        f.write("# CPU oracle on configuration 0 (B=8, Hq=4, Hkv=1, D=64, C=4 x L=256, k=2, U=128, f32), seed 20251106.\n")
        f.write("# Written by make_config0_golden.py from oracle/ only.  ids: routed chunks per (request, KV head);\n")
        f.write("# O / LSE: merged attention output of head 0 (first 8 dims) and log-sum-exp per request.\n")
        for b in range(p.B):
            f.write(f"ids {b} " + " ".join(str(int(c)) for c in st.ids[b, 0]) + "\n")
        for b in range(p.B):
            f.write(f"O {b} " + " ".join(f"{float(x):.17g}" for x in st.O_direct[b, 0, :8]) + "\n")
        for b in range(p.B):
            f.write(f"LSE {b} " + " ".join(f"{float(x):.17g}" for x in st.LSE_direct[b]) + "\n")


if __name__ == "__main__":
    main()
