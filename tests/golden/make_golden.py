"""Writes tests/golden/cfg1_oracle.txt from the CPU oracle alone (no GPU code is
called).  The paper prints no numeric example of the attention path, so this
fixture is not a citation: it freezes the oracle's own output on config 1 so
that an accidental change of the oracle's arithmetic or of the seeded input
recipe is noticed.  Re-run only together with a justified oracle change."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import tva_oracle as orc  # noqa: E402
from paper_2510_26577_amd import workloads as wl  # noqa: E402


def main():
    w = wl.config1()
    out, lse = orc.tree_verify_attn(w)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_oracle.txt")
    with open(path, "w") as f:
        f.write("# config 1 (B=1,Hq=Hkv=4,D=64,L=128,T=8), oracle output; written by make_golden.py\n")
        f.write("# parent: " + " ".join(str(int(p)) for p in w.parent) + "\n")
        f.write("# columns: node head lse out[0] out[1] out[62] out[63]\n")
        for i in range(8):
            for h in range(4):
                o = out[i, h]
                f.write(f"{i} {h} {lse[i, h]:.15e} {o[0]:.15e} {o[1]:.15e} {o[62]:.15e} {o[63]:.15e}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
