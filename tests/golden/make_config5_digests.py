"""Writes tests/golden/config5_digests.txt from the CPU oracle alone.

Run from the repository root (about 15 minutes on 8 cores):
    python tests/golden/make_config5_digests.py [--threads N]

Config 5 (B=128, k=64, V=50000, 120 steps) costs the oracle about 0.3 s per sentence and step,
too much to follow all 128 sentences inside a GPU test.  This script follows every sentence
through every step with the oracle and stores, per sentence, the chained digest (tests/digests.py)
of everything each step leaves behind, at every fifth step and at the last one, plus a digest of
what the end of decoding returns.  The GPU test feeds the HIP path's outputs of every step and
sentence into the same chains and compares them here; it also runs the oracle itself on a few
sentences and checks that those reproduce the stored values, so a table that no longer matches the
oracle or the input generator cannot go unnoticed.

The values are the oracle's, not the paper's (the paper prints no numeric example of a step).
Nothing here imports or runs the GPU library.
"""
import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))

import oracle  # noqa: E402
import synth_inputs as si  # noqa: E402
from digests import Chains, final_digest, write_table  # noqa: E402

EVERY = 5


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--threads", type=int, default=os.cpu_count() or 1)
    ap.add_argument("--steps", type=int, default=None, help="fewer steps, for a trial run (not for the stored table)")
    ap.add_argument("--out", default=os.path.join(HERE, "config5_digests.txt"))
    args = ap.parse_args()
    wl = si.make_config(5) if args.steps is None else si.make_config(5, T=args.steps)
    ob = oracle.BatchBeam(wl.k, wl.V, wl.constraints, wl.eos_id, wl.pad_id)
    chains = Chains(wl.B)
    steps = {}
    buf = np.empty((wl.B, wl.k, wl.V), dtype=np.float32)
    t0 = time.time()
    for t in range(wl.T):
        ob.step(wl.logp(t, out=buf), threads=args.threads)
        for i, bm in enumerate(ob.beams):
            chains.feed(i, dict(token=bm.token, backptr=bm.backptr, score=bm.score, flags=bm.flags,
                                met=bm.met, ip=bm.ip, iq=bm.iq, len=bm.len), bm.stop_bits)
        if t % EVERY == EVERY - 1 or t == wl.T - 1:
            steps[t] = chains.hex()
        print(f"step {t + 1}/{wl.T}  {time.time() - t0:.0f} s", flush=True)
    ft, fl, fs, fst = ob.finalize(wl.T)
    final = [final_digest(ft[b], fl[b], fs[b], fst[b]) for b in range(wl.B)]
    write_table(args.out,
                ["config 5 (B=128, k=64, V=50000, 120 steps), written by make_config5_digests.py from oracle/ only",
                 "line 't h0 h1 ...': chained digest of sentence 0, 1, ... after step t (0-based); 'final': end of decoding"],
                dict(config=5, seed=wl.seed, B=wl.B, k=wl.k, V=wl.V, T=wl.T, every=EVERY), steps, final)
    print("wrote", args.out)


if __name__ == "__main__":
    main()
