#!/usr/bin/env python3
"""Writes tests/golden/mbs_lut_fp16.txt: the 2 x 64 x 16 table of squared relative errors that MBS-Dynamic reads
(Sec. 4.3.3, Eq. 5), as fp16 bit patterns.  Every value comes from the CPU oracle (oracle.mbs_lut: the fp64
definition of an entry, rounded to fp16 by numpy); nothing here touches the HIP library.

Run from the repository root:  python tests/golden/make_mbs_lut.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402


def main():
    lut = oracle.mbs_lut()
    out = os.path.join(ROOT, "tests", "golden", "mbs_lut_fp16.txt")
    with open(out, "w") as f:
        f.write("# Table of Eq. 5 (Sec. 4.3.3): squared relative error of an element with scaled magnitude v under candidate\n")
        f.write("# word 16 j, fp16 bit patterns in hex.  One line per point: table (0 = sub-normal, v = (p + 1/2)/64;\n")
        f.write("# 1 = normal, v = 1 + (p + 1/2)/64), point p, then the 16 slots j = 0 .. 15.\n")
        f.write("# Written by tests/golden/make_mbs_lut.py from the CPU oracle; the paper gives the table's shape, not its values.\n")
        for t in range(2):
            for p in range(64):
                f.write("%d %2d %s\n" % (t, p, " ".join("%04x" % int(v) for v in lut[t, p])))
    print("wrote", out)


if __name__ == "__main__":
    main()
