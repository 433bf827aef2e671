"""Writes tests/golden/config1_trace.txt from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
The trace guards the oracle against silent change; it is not a value from the
paper (the paper prints no numeric worked example of a step).
Columns: step slot token parent score(fp32 bytes, hex) flags met-mask(hex)
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import synth_inputs as si  # noqa: E402


def main():
    wl = si.make_config(1)
    bm = oracle.SentenceBeam(wl.k, wl.V, wl.constraints[0], wl.eos_id, wl.pad_id)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_trace.txt")
    with open(out, "w") as fh:
        fh.write("# config 1 (B=1, k=5, V=1000, 20 steps), written by make_golden.py from oracle/ only\n")
        fh.write("# step slot token parent score_hex flags met_hex\n")
        for t in range(wl.T):
            bm.step(wl.logp(t)[0])
            for i in range(wl.k):
                fh.write("%d %d %d %d %s %d %x\n" % (
                    t, i, bm.token[i], bm.backptr[i], np.float32(bm.score[i]).tobytes().hex(),
                    bm.flags[i], int(bm.met[i])))


if __name__ == "__main__":
    main()
