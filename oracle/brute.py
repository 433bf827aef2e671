"""Brute-force enumerator of one DBA step, for tiny sizes only.

TEST INFRASTRUCTURE ONLY.  A second, deliberately differently-formulated
statement of Alg. 2 / Sections 3.1-3.3 of Post & Vilar (2018), used to
cross-check oracle/dba_oracle.c:
  * constraint state is a per-phrase progress counter, not per-token marks;
  * the expandable set is found by scanning EVERY vocabulary entry and asking
    "may hypothesis h place w now?", not by walking the phrase list;
  * the top-k is a stable full sort of the whole k x V matrix;
  * the bank of a candidate is recounted from its new state;
  * the allocation hands out slots one at a time to an explicitly sorted list
    of receivers.
It shares no code with the C oracle or with the GPU library.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


@dataclass
class Hyp:
    score: np.float32
    prog: List[int]                 # tokens met so far in every phrase (a prefix)
    active: Optional[int] = None    # phrase under way
    finished: bool = False
    length: int = 0

    def copy(self) -> "Hyp":
        return Hyp(self.score, list(self.prog), self.active, self.finished, self.length)


def met_mask(phrases, h: Hyp) -> int:
    m, base = 0, 0
    for j, ph in enumerate(phrases):
        for q in range(h.prog[j]):
            m |= 1 << (base + q)
        base += len(ph)
    return m


def may_place(phrases, h: Hyp, w: int) -> bool:
    """Is w one of the unmet constraint tokens hypothesis h can place next?"""
    for j, ph in enumerate(phrases):
        if h.prog[j] == len(ph):
            continue
        if h.active == j:
            if ph[h.prog[j]] == w:
                return True
        elif ph[0] == w:
            return True
    return False


def emit(phrases, h: Hyp, w: int) -> Hyp:
    """State of h after generating w (Sec. 3.1: in-order phrases, unwinding)."""
    n = h.copy()
    if n.active is not None:
        j = n.active
        if phrases[j][n.prog[j]] == w:
            n.prog[j] += 1
            if n.prog[j] == len(phrases[j]):
                n.active = None
            return n
        n.prog[j] = 0
        n.active = None
    for j, ph in enumerate(phrases):
        if n.prog[j] < len(ph) and ph[0] == w:
            n.prog[j] = 1
            if len(ph) > 1:
                n.active = j
            break
    return n


def allocate(k: int, cnt: List[int]) -> List[int]:
    """Slots per bank (Sec. 3.2), one slot at a time."""
    C = len(cnt) - 1
    share, rest = divmod(k, C + 1)
    alloc = [share] * (C + 1)
    alloc[C] += rest
    for b in range(C + 1):
        spare = alloc[b] - cnt[b]
        if spare <= 0:
            continue
        alloc[b] = cnt[b]
        receivers = sorted((x for x in range(C + 1) if x != b), key=lambda x: (abs(x - b), -x))
        for x in receivers:
            while spare > 0 and alloc[x] < cnt[x]:
                alloc[x] += 1
                spare -= 1
    return alloc


def step(beam: List[Optional[Hyp]], logp: np.ndarray, phrases, eos_id: int, pad_id: int,
         adjust: bool = True, normalize: bool = False, prune: Optional[float] = None
         ) -> Tuple[List[Optional[Tuple[int, int, Hyp]]], dict]:
    """One step.  beam[h] is None for an empty slot.  Returns the new beam as
    (token, parent, hypothesis) triples best first (None = empty slot) and a
    dict of intermediate facts.  adjust=False: bank sizes stay at the base split
    (Sec. 5); normalize: a hypothesis completing now is stored with sum/length
    (Sec. 4); prune: hypotheses below best-completed minus this are struck out
    (Sec. 4, Sec. 6.3)."""
    k, V = logp.shape
    C = sum(len(p) for p in phrases)
    s = np.full((k, V), -np.inf, dtype=np.float32)
    for h, hyp in enumerate(beam):
        if hyp is None:
            continue
        if hyp.finished:
            s[h, pad_id] = np.float32(hyp.score) + np.float32(0.0)
            continue
        s[h] = np.float32(hyp.score) + logp[h].astype(np.float32)
        if sum(hyp.prog) < C:
            s[h, eos_id] = -np.inf
    flat_s = s.reshape(-1)
    order = np.argsort(-flat_s.astype(np.float64), kind="stable")
    cands = set()
    for f in order[:k]:
        if flat_s[f] > -np.inf:
            cands.add(int(f))
    topk = sorted(cands)
    for h, hyp in enumerate(beam):
        if hyp is None:
            continue
        if not hyp.finished:
            for w in range(V):
                if may_place(phrases, hyp, w) and s[h, w] > -np.inf:
                    cands.add(h * V + w)
        best = int(np.flatnonzero(s[h] == s[h].max())[0])
        if s[h, best] > -np.inf:
            cands.add(h * V + best)
    items = []
    for f in sorted(cands):
        h, w = divmod(f, V)
        parent = beam[h]
        new = parent.copy() if parent.finished else emit(phrases, parent, w)
        if not parent.finished:
            new.length = parent.length + 1
            new.finished = (w == eos_id)
        new.score = s[h, w]
        items.append((sum(new.prog), float(s[h, w]), f, w, h, new))
    cnt = [0] * (C + 1)
    for it in items:
        cnt[it[0]] += 1
    if adjust:
        alloc = allocate(k, cnt)
    else:
        share, rest = divmod(k, C + 1)
        alloc = [min(cnt[b], share + (rest if b == C else 0)) for b in range(C + 1)]
    chosen = []
    for b in range(C + 1):
        members = sorted((it for it in items if it[0] == b), key=lambda it: (-it[1], it[2]))
        chosen.extend(members[:alloc[b]])
    chosen.sort(key=lambda it: (-it[1], it[2]))
    out: List[Optional[Tuple[int, int, Hyp]]] = [(it[3], it[4], it[5]) for it in chosen]
    if normalize:
        for w, h, new in out:
            if new.finished and not beam[h].finished:
                new.score = np.float32(new.score) / np.float32(new.length)
    if prune is not None:
        done = [np.float32(new.score) for _, _, new in out if new.finished]
        if done:
            cut = np.float32(max(done)) - np.float32(prune)
            out = [x for x in out if not np.float32(x[2].score) < cut]
    stop = bool(out) and all(new.finished for _, _, new in out)
    some = any(new.finished for _, _, new in out)
    out += [None] * (k - len(out))
    return out, dict(cands=sorted(cands), topk=topk, cnt=cnt, alloc=alloc, all_finished=stop, any_finished=some)
