"""Writes tests/golden/cfg0_expected.txt from the float64 oracle alone.

Run from the repository root:  python tests/golden/make_cfg0_expected.py
Calls only oracle/ and the seeded input generator.  The stored values guard
the oracle against accidental change; they are not values printed by the
paper (it prints none for this layer).
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import attn_ref  # noqa: E402
from paper_1805_08899_amd.workloads import WORKLOADS, make_inputs  # noqa: E402


def main():
    d = make_inputs(WORKLOADS[0])
    out = attn_ref.forward_backward(d["Qp"], d["Kp"], d["V"], d["v"], d["key_len"], d["dContext"])
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg0_expected.txt")
    with open(path, "w") as f:
        f.write("# float64 oracle outputs for workload 0 (B=4,Tq=6,Tk=7,H=16,Dv=16), default seed\n")
        f.write("# written by tests/golden/make_cfg0_expected.py; one tensor per block: name, shape, values\n")
        f.write("key_len " + " ".join(str(int(x)) for x in d["key_len"]) + "\n")
        for k in ("context", "P", "dQp", "dKp", "dV", "dv"):
            a = out[k]
            f.write(f"{k} {' '.join(str(s) for s in a.shape)}\n")
            f.write(" ".join(repr(float(x)) for x in a.ravel()) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
