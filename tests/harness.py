"""GPU-vs-oracle comparison used by the gpu tests: the HIP path (through the C ABI) and the
CPU oracle get the same seeded log-prob bytes, step after step, and every output is compared
element by element - bit-exact for tokens, parents, flags, constraint state AND fp32 scores
(a score is one fp32 add on both sides)."""
from __future__ import annotations

import os
from typing import Optional, Sequence

import numpy as np
import torch

import digests
import oracle
import synth_inputs as si
from paper_1804_06609_amd.session import Session

THREADS = min(16, os.cpu_count() or 1)


def _first_diff(name, got, want, t, sent_ids):
    if got.tobytes() == want.tobytes():
        return
    bad = np.argwhere(got.view(np.uint8).reshape(got.shape + (-1,)).astype(np.int16) !=
                      want.view(np.uint8).reshape(want.shape + (-1,)).astype(np.int16))
    i, h = int(bad[0][0]), int(bad[0][1])
    raise AssertionError(
        f"{name} differs at step {t}, sentence {sent_ids[i]}, slot {h}: "
        f"gpu={got[i, h]!r} oracle={want[i, h]!r}\n gpu row   : {got[i]}\n oracle row: {want[i]}")


def run_parity(wl: si.Workload, T: Optional[int] = None, oracle_sentences: Optional[Sequence[int]] = None,
               check_state_every: int = 1, check_invariants: bool = True, progress: str = "",
               options: Optional[dict] = None, adjust: bool = True, normalize: bool = False,
               prune: Optional[float] = None, logp_format: Optional[str] = None,
               golden: Optional[str] = None, track: bool = False):
    """Runs T steps of wl on the GPU and on the oracle (all sentences, or the sampled ones) and
    compares every step.  Returns the session's finalize() result after checking it too.
    golden: a table of chained digests written by the oracle beforehand for ALL sentences
    (tests/golden/make_config5_digests.py): the GPU outputs of every sentence and step are fed
    into the same chains and compared at every stored step; the sentences the oracle follows
    live must reproduce the table too.  A sentence that disagrees is re-run on the oracle from
    the first step to name the element.
    adjust / normalize / prune switch the same variant on both sides (Sec. 5; Sec. 4); so does track
    (the best completed hypothesis seen on any beam is remembered and returned at the end, Sec. 3.3).
    logp_format "f16" / "bf16": the generator's log-probs are rounded once more to that type; the
    GPU gets the 16-bit tensor, the oracle the same values widened (exactly) to fp32."""
    import paper_1804_06609_amd as dba
    options = dict(options or {})
    options[dba.DBA_OPT_ADJUSTMENT] = int(adjust)
    options[dba.DBA_OPT_NORMALIZE_FINISHED] = int(normalize)
    options[dba.DBA_OPT_PRUNE_THRESHOLD] = -1.0 if prune is None else prune
    options[dba.DBA_OPT_TRACK_COMPLETED] = int(track)
    T = wl.T if T is None else T
    B, k, V = wl.B, wl.k, wl.V
    sent = list(range(B)) if oracle_sentences is None else sorted(oracle_sentences)
    toks, poff, soff = wl.csr()
    ses = Session(B, k, V, T, wl.eos_id, wl.pad_id, toks, poff, soff, options=options)
    ob = oracle.BatchBeam(k, V, wl.constraints, wl.eos_id, wl.pad_id, sentences=sent, adjust=adjust,
                          normalize_finished=normalize, prune_threshold=prune, track_completed=track)
    g_chain = o_chain = None
    if golden:
        head, g_steps, g_final = digests.read_table(golden)
        assert (int(head["B"]), int(head["k"]), int(head["V"]), int(head["seed"])) == (B, k, V, wl.seed), head
        assert logp_format is None and adjust and not normalize and prune is None
        g_chain, o_chain = digests.Chains(B), digests.Chains(len(sent))
        recent = []                       # GPU outputs since the last stored step
        last_stored = -1
    host = torch.empty((B, k, V), dtype=torch.float32, pin_memory=True)
    tdt = {None: torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[logp_format]
    dev = torch.empty((B, k, V), dtype=tdt, device="cuda")
    for t in range(T):
        lp = wl.logp(t, out=host.numpy())
        if logp_format is None:
            dev.copy_(host, non_blocking=False)
        else:
            bits = si.narrow16(lp, logp_format)
            dev.copy_(torch.from_numpy(bits.view(np.int16)).view(tdt))
            lp = oracle.widen16(bits, logp_format)
        ses.step(dev)
        ob.step(lp[sent], threads=THREADS)
        g_tok, g_bp, g_sc, g_fl = ses.outputs()
        _first_diff("token", g_tok[sent], ob.stacked("token"), t, sent)
        _first_diff("backptr", g_bp[sent], ob.stacked("backptr"), t, sent)
        _first_diff("score", g_sc[sent], ob.stacked("score"), t, sent)
        _first_diff("flags", g_fl[sent], ob.stacked("flags"), t, sent)
        st = None
        if golden or (check_state_every and (t % check_state_every == 0 or t == T - 1)):
            st = ses.state()
        if st is not None:
            _first_diff("state.score", st["score"][sent], ob.stacked("score"), t, sent)
            _first_diff("state.met", st["met_mask"][sent], ob.stacked("met"), t, sent)
            _first_diff("state.inprog_phrase", st["inprog_phrase"][sent], ob.stacked("ip"), t, sent)
            _first_diff("state.inprog_pos", st["inprog_pos"][sent], ob.stacked("iq"), t, sent)
            _first_diff("state.length", st["length"][sent], ob.stacked("len"), t, sent)
            _first_diff("state.flags", st["flags"][sent], ob.stacked("flags"), t, sent)
        done = ses.finished()
        assert done[sent].tolist() == [bm.stop_bits for bm in ob.beams], f"stopping flags, step {t}"
        if golden:
            assert st["score"].tobytes() == g_sc.tobytes() and st["flags"].tobytes() == g_fl.tobytes(), t
            gpu_fields = dict(token=g_tok, backptr=g_bp, score=g_sc, flags=g_fl, met=st["met_mask"],
                              ip=st["inprog_phrase"], iq=st["inprog_pos"], len=st["length"])
            recent.append((t, gpu_fields, done.copy()))
            for b in range(B):
                g_chain.feed(b, {n: a[b] for n, a in gpu_fields.items()}, done[b])
            for i, bm in enumerate(ob.beams):
                o_chain.feed(i, dict(token=bm.token, backptr=bm.backptr, score=bm.score, flags=bm.flags,
                                     met=bm.met, ip=bm.ip, iq=bm.iq, len=bm.len), bm.stop_bits)
            if t in g_steps:
                want = g_steps[t]
                live = o_chain.hex()
                for i, b in enumerate(sent):
                    assert live[i] == want[b], (
                        f"the stored digests are not what the oracle computes now (step {t}, sentence {b}): "
                        f"run tests/golden/make_config5_digests.py again")
                bad = [b for b, h in enumerate(g_chain.hex()) if h != want[b]]
                if bad:
                    _explain(wl, bad[0], last_stored, t, recent)
                recent = []
                last_stored = t
        if check_invariants:
            check_step_properties(wl, g_tok, g_bp, g_sc, g_fl, ordered=not normalize)
        if progress and (t % 10 == 9 or t == T - 1):
            print(f"  {progress}: step {t + 1}/{T} ok", flush=True)
    fin = ses.finalize()
    o_fin = ob.finalize(T)
    for name, g, o in zip(("final tokens", "final len", "final score", "final status"), fin, o_fin):
        assert g[sent].tobytes() == o.tobytes(), name
    if golden and T == int(head["T"]):
        assert last_stored == T - 1
        got = [digests.final_digest(fin[0][b], fin[1][b], fin[2][b], fin[3][b]) for b in range(B)]
        bad = [b for b in range(B) if got[b] != g_final[b]]
        assert not bad, f"end of decoding differs from the oracle's stored digest for sentences {bad}"
    ses.close()
    return fin


def _explain(wl, b, t_ok, t_bad, recent):
    """Sentence b agreed with the oracle's stored digest after step t_ok and not after t_bad: run the
    oracle on it from the first step and name the first element that differs."""
    bm = oracle.SentenceBeam(wl.k, wl.V, wl.constraints[b], wl.eos_id, wl.pad_id)
    by_step = {t: (f, d) for t, f, d in recent}
    for t in range(t_bad + 1):
        bm.step(wl.logp(t, sentences=[b])[0])
        if t <= t_ok:
            continue
        f, done = by_step[t]
        for name, want in (("token", bm.token), ("backptr", bm.backptr), ("score", bm.score), ("flags", bm.flags),
                           ("met", bm.met), ("ip", bm.ip), ("iq", bm.iq), ("len", bm.len)):
            _first_diff(name, f[name][b:b + 1], want[None, :], t, [b])
        assert int(done[b]) == bm.stop_bits, f"stopping flags of sentence {b} at step {t}"
    raise AssertionError(f"sentence {b}: digest differs between steps {t_ok + 1} and {t_bad}, "
                         f"but the oracle re-run agrees element by element (stale table?)")


def check_step_properties(wl, tok, bp, sc, fl, ordered=True):
    """Properties of one step's output that hold for every sentence at any size."""
    live = fl != 2
    assert ((sc == -np.inf) == ~live).all()
    assert (bp[~live] == -1).all() and (tok[~live] == wl.pad_id).all()
    assert ((bp[live] >= 0) & (bp[live] < wl.k)).all()
    assert ((tok[live] >= 0) & (tok[live] < wl.V)).all()
    # live slots come first and are in non-increasing score order
    assert (live[:, :-1] >= live[:, 1:]).all()
    s2 = np.where(live, sc, -np.inf)
    assert not ordered or (s2[:, :-1] >= s2[:, 1:]).all()
    # no coordinate twice in a beam
    flat = np.where(live, bp.astype(np.int64) * wl.V + tok, -1 - np.arange(wl.k)[None, :])
    srt = np.sort(flat, axis=1)
    assert (srt[:, 1:] != srt[:, :-1]).all()
