#!/usr/bin/env python3
"""Alg. 1 of Post & Vilar (2018) around libdba, with a stand-in decoder.

The "decoder" here is the seeded synthetic generator (per-step log-probs that do not depend on the
beam); a real decoder would run its network on the beam returned by the previous step - the
tokens in `ses.out_token`, re-ordered by `ses.out_backptr` - and hand over its [B, k, V] log-probs,
which never have to leave the GPU.  Shows the settings of the paper's experiments (Sec. 4):
per-word scores for completed hypotheses, pruning threshold 20, stop when every hypothesis on the
beam is completed.

    python examples/decode_loop.py [--batch 8] [--beam 10] [--vocab 32000] [--max-len 60]
"""
from __future__ import annotations

import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--beam", type=int, default=10)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--max-len", type=int, default=60)
    args = ap.parse_args()

    import torch
    import paper_1804_06609_amd as dba
    import synth_inputs as si
    from paper_1804_06609_amd.session import Session

    B, k, V, N = args.batch, args.beam, args.vocab, args.max_len
    # constraints: for every sentence 1..4 phrases of 1..3 tokens (word and phrasal constraints, Sec. 3)
    wl = si.make_small(2018, B, k, V, N, max_phrases=4, max_len=3, dup_prob=0.0)
    wl.eos_switch = N // 3                       # the stand-in decoder starts to like end-of-sentence here
    toks, poff, soff = wl.csr()
    ses = Session(B, k, V, N, wl.eos_id, wl.pad_id, toks, poff, soff, options={
        dba.DBA_OPT_NORMALIZE_FINISHED: 1, dba.DBA_OPT_PRUNE_THRESHOLD: 20.0,
        dba.DBA_OPT_TRACK_COMPLETED: 1})         # Sec. 3.3: the best completed hypothesis, also if it has left the beam

    steps = 0
    for t in range(N):                           # Alg. 1: for time step t in 1..N
        logp = torch.from_numpy(wl.logp(t)).cuda()       # decoder-step (stand-in)
        ses.step(logp)                           # kbest-DBA (Alg. 2)
        steps += 1
        if (ses.finished() & dba.DBA_STOP_ALL).all():    # Sec. 4: every hypothesis is completed
            break
    tokens, length, score, status = ses.finalize()
    print(f"{steps} steps")
    for b in range(B):
        cons = " | ".join(" ".join(map(str, p)) for p in wl.constraints[b]) or "-"
        out = " ".join(map(str, tokens[b, :length[b]]))
        print(f"sentence {b}: constraints [{cons}]  status {status[b]}  score/word {score[b]:.3f}\n  {out}")
    ses.close()


if __name__ == "__main__":
    main()
