"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each is chosen so that a
plausible slip in oracle/dba_oracle.c (dropped candidate source, wrong tie
rule, wrong neighbour order, missed unwinding, EOS let through) fails it.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import brute
import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------
# allocation (Sec. 3.2)
# --------------------------------------------------------------------------
def _figure_rows():
    rows = []
    with open(os.path.join(GOLDEN, "figure_allocation_facts.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            src, k, C, cnt, facts = [x.strip() for x in line.split("|")]
            rows.append((src, int(k), int(C), [int(x) for x in cnt.split()], facts))
    return rows


@pytest.mark.parametrize("src,k,C,cnt,facts", _figure_rows())
def test_allocation_figure_facts(src, k, C, cnt, facts):
    """Fig. 2 and Fig. 3 captions: k=5, four constraints."""
    assert len(cnt) == C + 1
    alloc = oracle.allocate(k, cnt)
    for fact in [f.strip() for f in facts.split(";")]:
        if fact.startswith("alloc ="):
            assert list(alloc) == [int(x) for x in fact.split("=")[1].split()]
        elif fact.startswith("sum ="):
            assert int(alloc.sum()) == int(fact.split("=")[1])
        elif fact.startswith("alloc[2..4] = 0"):
            assert list(alloc[2:5]) == [0, 0, 0]
        elif fact == "alloc <= count":
            assert all(a <= c for a, c in zip(alloc, cnt))
        else:
            raise AssertionError("unknown fact " + fact)


def test_allocation_invariants_exhaustive():
    """Sec. 3.2: the beam is filled up to min(k, #candidates); no bank gets more
    than it can fill; a bank that can fill its base share keeps at least that;
    with no constraints there is one bank of k (plain beam search)."""
    n = 0
    for k in range(1, 8):
        for C in range(0, 5):
            base = [k // (C + 1)] * (C + 1)
            base[C] += k % (C + 1)
            for cnt in itertools.product(range(0, k + 2), repeat=C + 1):
                alloc = oracle.allocate(k, cnt)
                assert int(alloc.sum()) == min(k, sum(cnt)), (k, cnt, alloc)
                assert all(0 <= a <= c for a, c in zip(alloc, cnt)), (k, cnt, alloc)
                assert all(a >= min(c, b) for a, c, b in zip(alloc, cnt, base)), (k, cnt, alloc)
                assert list(alloc) == brute.allocate(k, list(cnt)), (k, cnt, alloc)
                n += 1
    assert n > 50000


def test_allocation_more_constraints_than_slots():
    """Sec. 5: adjustment lets DBA work when C >= k (k=5 shown).  With C >= k
    every base share is 0 and all k slots start at the topmost bank, so the
    slots end up in the highest non-empty banks."""
    k, C = 5, 32
    cnt = [0] * (C + 1)
    cnt[0], cnt[1], cnt[2] = 9, 2, 1
    alloc = oracle.allocate(k, cnt)
    assert list(alloc[:3]) == [2, 2, 1] and int(alloc.sum()) == k
    cnt = [0] * (C + 1)
    cnt[32], cnt[30], cnt[7] = 1, 1, 40
    alloc = oracle.allocate(k, cnt)
    assert alloc[32] == 1 and alloc[30] == 1 and alloc[7] == 3


def test_allocation_neighbour_order():
    """The reading of 'immediate neighbours first, moving outward': distance 1
    before distance 2, and at equal distance the higher bank is served first."""
    # k=6, C=2: base 2,2,2.  Bank 1 is empty: its 2 slots go to bank 2 first.
    assert list(oracle.allocate(6, [5, 0, 5])) == [2, 0, 4]
    # bank 2 can only take one more: the second slot goes down to bank 0
    assert list(oracle.allocate(6, [5, 0, 3])) == [3, 0, 3]
    # k=8, C=3: base 2 each.  Bank 0 empty: nearest taker is bank 1, then bank 2.
    assert list(oracle.allocate(8, [0, 3, 9, 2])) == [0, 3, 3, 2]


# --------------------------------------------------------------------------
# constraint bookkeeping (Sec. 3.1)
# --------------------------------------------------------------------------
def test_add_phrase_in_order_and_unwinding():
    a, b, c, d = 11, 12, 13, 14
    phrases = [[a, b], [c]]           # a phrasal constraint of length 2 and a word (cf. Fig. 2)
    # nothing met: expandable = first token of the phrase, and the word
    met, ip, iq, nxt = oracle.add(phrases, 0, -1, 0, -1)
    assert (met, ip, iq) == (0, -1, 0) and nxt == [a, c]
    # second half alone does nothing: phrases complete in order only
    assert oracle.add(phrases, 0, -1, 0, b)[:3] == (0, -1, 0)
    # first half: met, phrase under way
    met, ip, iq, _ = oracle.add(phrases, 0, -1, 0, a)
    assert (met, ip, iq) == (0b001, 0, 1)
    # now expandable = the second half, and the word
    assert oracle.add(phrases, met, ip, iq, -1)[3] == [b, c]
    # second half completes it
    assert oracle.add(phrases, met, ip, iq, b)[:3] == (0b011, -1, 0)
    # anything else unwinds the first half (Sec. 3.1, last paragraph)
    assert oracle.add(phrases, met, ip, iq, d)[:3] == (0, -1, 0)
    # ... even a token that meets another constraint: the phrase is unwound, the word is met
    assert oracle.add(phrases, met, ip, iq, c)[:3] == (0b100, -1, 0)
    # the first half again: unwound and begun anew
    assert oracle.add(phrases, met, ip, iq, a)[:3] == (0b001, 0, 1)
    # a completed phrase is never unwound or re-counted
    assert oracle.add(phrases, 0b011, -1, 0, a)[:3] == (0b011, -1, 0)
    assert oracle.add(phrases, 0b011, -1, 0, d)[:3] == (0b011, -1, 0)
    assert oracle.add(phrases, 0b011, -1, 0, -1)[3] == [c]
    assert oracle.add(phrases, 0b111, -1, 0, -1)[3] == []


def test_add_repeated_tokens():
    a, b = 21, 22
    # the same word twice: two obligations, one emitted token meets one of them
    phrases = [[a], [a]]
    m1 = oracle.add(phrases, 0, -1, 0, a)
    assert m1[:3] == (0b01, -1, 0)
    assert oracle.add(phrases, 0b01, -1, 0, a)[:3] == (0b11, -1, 0)
    assert oracle.add(phrases, 0b01, -1, 0, -1)[3] == [a]
    # phrases sharing a first token: the lower phrase index is begun
    phrases = [[a, b], [a]]
    assert oracle.add(phrases, 0, -1, 0, a)[:3] == (0b001, 0, 1)
    # while [a b] is under way, 'a' breaks it, unwinds it and starts it again
    assert oracle.add(phrases, 0b001, 0, 1, a)[:3] == (0b001, 0, 1)
    # once [a b] is complete, 'a' meets the word
    assert oracle.add(phrases, 0b011, -1, 0, a)[:3] == (0b111, -1, 0)
    # a phrase whose tokens repeat: a a b
    phrases = [[a, a, b]]
    s1 = oracle.add(phrases, 0, -1, 0, a)[:3]
    s2 = oracle.add(phrases, *s1, a)[:3]
    assert s1 == (0b001, 0, 1) and s2 == (0b011, 0, 2)
    # a third 'a' breaks it: full reset, then begun anew (no partial fallback)
    assert oracle.add(phrases, *s2, a)[:3] == (0b001, 0, 1)
    assert oracle.add(phrases, *s2, b)[:3] == (0b111, -1, 0)


# --------------------------------------------------------------------------
# whole step
# --------------------------------------------------------------------------
def _textbook_topk_step(prev, fin, logp, k, pad_id):
    """Plain beam search step: sorted top-k of the k x V matrix of sums."""
    s = (prev[:, None] + logp).astype(np.float32)
    for h in range(len(prev)):
        if fin[h]:
            s[h] = -np.inf
            s[h, pad_id] = prev[h]
    order = np.argsort(-s.reshape(-1).astype(np.float64), kind="stable")[:k]
    order = [f for f in order if s.reshape(-1)[f] > -np.inf]
    return order, s.reshape(-1)[order]


@pytest.mark.parametrize("k,V", [(1, 50), (5, 1000), (10, 4000)])
def test_no_constraints_is_plain_beam_search(k, V):
    """Sec. 3: with no constraints kbest-DBA is the ordinary top-k of the scores
    matrix; here checked step after step, indices and fp32 scores exactly."""
    T = 30
    wl = si.Workload(B=1, k=k, V=V, T=T, seed=77, constraints=[[]], eos_switch=12)
    bm = oracle.SentenceBeam(k, V, [], wl.eos_id, wl.pad_id)
    for t in range(T):
        logp = wl.logp(t)[0]
        fin = (bm.flags & oracle.FLAG_FINISHED) != 0
        flat, sc = _textbook_topk_step(bm.score.copy(), fin, logp, k, wl.pad_id)
        bm.step(logp)
        n = len(flat)
        assert list(bm.backptr[:n] * V + bm.token[:n]) == [int(f) for f in flat]
        assert bm.score[:n].tobytes() == np.asarray(sc, np.float32).tobytes()
        assert all(bm.flags[n:] == oracle.FLAG_DEAD)
    assert (bm.flags & oracle.FLAG_FINISHED).any()     # the EOS schedule did finish something


def test_equal_scores_go_to_the_lower_coordinate():
    """Ties: two rows with identical sums; the lower flat coordinate wins everywhere."""
    k, V = 3, 8
    logp = np.full((k, V), -5.0, dtype=np.float32)
    logp[:, 4] = -1.0
    logp[:, 6] = -1.0
    bm = oracle.SentenceBeam(k, V, [], 2, 0)
    bm.score[:] = 0.0
    bm.flags[:] = 0
    bm.step(logp)
    assert list(bm.backptr) == [0, 0, 1] and list(bm.token) == [4, 6, 4]
    # sums that tie only after rounding: 2^24 - 0.5 and 2^24 - 0.25 both round to 2^24, so the
    # comparison is on the fp32 sums and entry 3 wins although entry 5 has the larger log-prob
    logp = np.full((1, V), -3.0, dtype=np.float32)
    logp[0, 3] = -0.5
    logp[0, 5] = -0.25
    bm = oracle.SentenceBeam(1, V, [], 2, 0)
    bm.score[0] = np.float32(2.0 ** 24)
    bm.step(logp)
    assert bm.token[0] == 3 and bm.score[0] == np.float32(2.0 ** 24)


def test_row_best_tie_goes_to_the_lower_token():
    """Sec. 3.1 item 3 under ties: a row's single best is its lowest-index maximum, also when
    that row does not reach the overall top-k."""
    k, V = 2, 8
    logp = np.full((k, V), -9.0, dtype=np.float32)
    logp[0, 1] = logp[0, 2] = -1.0          # fill the overall top-k from row 0
    logp[1, 5] = logp[1, 7] = -4.0          # row 1: two equal maxima
    bm = oracle.SentenceBeam(k, V, [], 3, 0)
    bm.score[:] = 0.0
    bm.flags[:] = 0
    bm.step(logp, debug=True)
    assert sorted(bm.dbg["flat"].tolist()) == [1, 2, V + 5]


def _brute_beam_init(k, phrases):
    beam = [None] * k
    beam[0] = brute.Hyp(np.float32(0.0), [0] * len(phrases))
    return beam


def _compare_with_brute(bm, new, phrases, k, pad_id):
    for i, item in enumerate(new):
        if item is None:
            assert bm.flags[i] == oracle.FLAG_DEAD and bm.backptr[i] == -1
            assert bm.token[i] == pad_id and bm.score[i] == -np.inf
            continue
        w, h, hyp = item
        assert (int(bm.token[i]), int(bm.backptr[i])) == (w, h)
        assert np.float32(bm.score[i]).tobytes() == np.float32(hyp.score).tobytes()
        assert int(bm.met[i]) == brute.met_mask(phrases, hyp)
        assert int(bm.ip[i]) == (-1 if hyp.active is None else hyp.active)
        assert int(bm.iq[i]) == (0 if hyp.active is None else hyp.prog[hyp.active])
        assert bool(bm.flags[i] & oracle.FLAG_FINISHED) == hyp.finished
        assert int(bm.len[i]) == hyp.length


@pytest.mark.parametrize("seed", range(120))
def test_oracle_matches_brute_force(seed):
    """Tiny shapes, repeated tokens, shared prefixes, boosted constraint tokens
    (so phrases start, break and finish), EOS switched on half way."""
    rs = si.Stream(seed, 99)
    k = rs.randint(1, 5)
    V = rs.randint(6, 40)
    T = rs.randint(4, 10)
    wl = si.make_small(seed, 1, k, V, T, max_phrases=4, max_len=3, dup_prob=0.4)
    wl.eos_switch = T // 2
    phrases = wl.constraints[0]
    bm = oracle.SentenceBeam(k, V, phrases, wl.eos_id, wl.pad_id)
    beam = _brute_beam_init(k, phrases)
    for t in range(T):
        logp = wl.logp(t)[0]
        new, info = brute.step(beam, logp, phrases, wl.eos_id, wl.pad_id)
        bm.step(logp, debug=True)
        assert sorted(int(f) for f in bm.dbg["flat"]) == info["cands"]
        assert list(bm.dbg["cnt"]) == info["cnt"]
        assert list(bm.dbg["alloc"]) == info["alloc"]
        _compare_with_brute(bm, new, phrases, k, wl.pad_id)
        beam = [None if it is None else it[2] for it in new]


def _check_trajectory(wl, b, T, debug_every=1):
    k, V = wl.k, wl.V
    phrases = wl.constraints[b]
    C = sum(len(p) for p in phrases)
    bm = oracle.SentenceBeam(k, V, phrases, wl.eos_id, wl.pad_id)
    seen_unwind = seen_finish = 0
    for t in range(T):
        logp = wl.logp(t, sentences=[b])[0]
        p_score, p_met, p_ip, p_iq, p_flags = (bm.score.copy(), bm.met.copy(), bm.ip.copy(),
                                               bm.iq.copy(), bm.flags.copy())
        p_nmet = bm.nmet
        bm.step(logp, debug=True)
        d = bm.dbg
        ncand = len(d["flat"])
        live = bm.flags != oracle.FLAG_DEAD
        # Sec. 3.2: filled up to min(k, #candidates); no bank over its count
        assert int(d["alloc"].sum()) == min(k, ncand) == int(live.sum())
        assert (d["alloc"] <= d["cnt"]).all()
        assert len(set(d["flat"].tolist())) == ncand
        # Sec. 3.1: the beam is kept best first
        sc = bm.score[live]
        assert (sc[:-1] >= sc[1:]).all()
        # item 1 of Sec. 3.1: the k best of the matrix are candidates
        s = (p_score[:, None] + logp).astype(np.float32)
        for h in range(k):
            if p_flags[h] & oracle.FLAG_FINISHED:
                s[h] = -np.inf
                s[h, wl.pad_id] = p_score[h]
            elif p_nmet[h] < C:
                s[h, wl.eos_id] = -np.inf
        top = np.argsort(-s.reshape(-1).astype(np.float64), kind="stable")[:k]
        top = [int(f) for f in top if s.reshape(-1)[f] > -np.inf]
        assert set(top) <= set(d["flat"].tolist())
        # item 3: every live row's best entry is a candidate
        for h in range(k):
            if p_score[h] > -np.inf:
                assert h * V + int(np.argmax(s[h])) in set(d["flat"].tolist())
        # inside a bank the chosen ones are the best of that bank
        sel = set((bm.backptr[live] * V + bm.token[live]).tolist())
        for bank in range(C + 1):
            members = [int(f) for f, bk in zip(d["flat"], d["bank"]) if bk == bank]
            members.sort(key=lambda f: (-float(s.reshape(-1)[f]), f))
            picked = [f in sel for f in members]
            assert picked == sorted(picked, reverse=True)
            assert sum(picked) == d["alloc"][bank]
        nm = bm.nmet
        for i in np.flatnonzero(live):
            h, w = int(bm.backptr[i]), int(bm.token[i])
            fin = bool(bm.flags[i] & oracle.FLAG_FINISHED)
            if fin:
                assert nm[i] == C                      # Sec. 3.3
                seen_finish += 1
            if nm[i] < p_nmet[h]:                      # only a broken phrase loses tokens
                assert p_ip[h] >= 0
                nxt = phrases[p_ip[h]][p_iq[h]]
                assert w != nxt and p_nmet[h] - nm[i] <= p_iq[h]
                seen_unwind += 1
            else:
                assert nm[i] - p_nmet[h] <= 1
            assert bm.score[i] == s[h, w]
    return seen_unwind, seen_finish


def test_trajectory_invariants_config1():
    wl = si.make_config(1)
    _check_trajectory(wl, 0, wl.T)


def test_trajectory_invariants_boosted_phrases():
    """Config-3-like sentences (boosted constraint tokens start and break phrases)."""
    wl = si.make_config(3, T=40)
    wl.V = 2000                                        # same recipe, smaller vocabulary for speed
    wl.constraints = [[[4 + (w % (wl.V - 4)) for w in ph] for ph in s] for s in wl.constraints]
    wl.boost_tokens = [[4 + (w % (wl.V - 4)) for w in s] for s in wl.boost_tokens]
    wl._zb = None
    unw = fin = 0
    for b in (0, 1, 2, 3):
        u, f = _check_trajectory(wl, b, 40)
        unw += u
        fin += f
    assert fin > 0


def test_unwinding_and_finishing_are_exercised():
    """The small fuzz recipe must actually reach unwinding and finishing."""
    unw = fin = 0
    for seed in range(40):
        wl = si.make_small(1000 + seed, 1, 4, 30, 10, max_phrases=3, max_len=3, dup_prob=0.4)
        wl.eos_switch = 5
        u, f = _check_trajectory(wl, 0, 10)
        unw += u
        fin += f
    assert unw > 0 and fin > 0


def test_finalize_picks_best_length_normalised_completed():
    """Sec. 3.3 / Sec. 4: the best completed hypothesis, scores divided by length."""
    k, T, N, pad = 3, 4, 6, 0
    ht = np.array([[5, 6, 7], [8, 2, 9], [0, 0, 2], [0, 0, 0]], np.int32)   # EOS id 2
    hb = np.array([[0, 0, 0], [0, 1, 2], [1, 0, 2], [0, 1, 2]], np.int32)
    bm = oracle.SentenceBeam(k, 10, [], 2, pad)
    bm.hist_token = list(ht)
    bm.hist_backptr = list(hb)
    # final slots: 0 <- finished at len 2 (tokens 6,2), 1 <- unfinished, 2 <- finished at len 3 (7,9,2)
    bm.score = np.array([-3.0, -1.0, -3.9], np.float32)
    bm.flags = np.array([1, 0, 1], np.uint8)
    bm.len = np.array([2, 4, 3], np.int32)
    toks, ln, sc, status = bm.finalize(N)
    # -3.0/2 = -1.5 < -3.9/3 = -1.3: slot 2 wins although its raw score is lower
    assert status == 1 and ln == 3 and sc == np.float32(-3.9)
    assert list(toks) == [7, 9, 2, 0, 0, 0]
    bm.flags = np.array([0, 0, 0], np.uint8)           # nobody completed
    bm.len = np.array([4, 4, 4], np.int32)
    toks, ln, sc, status = bm.finalize(N)
    assert status == 0 and ln == 4 and sc == np.float32(-1.0)
    assert list(toks) == [5, 8, 0, 0, 0, 0]


def test_golden_trace_config1():
    """Stored trace written by tests/golden/make_golden.py (oracle only)."""
    path = os.path.join(GOLDEN, "config1_trace.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    wl = si.make_config(1)
    bm = oracle.SentenceBeam(wl.k, wl.V, wl.constraints[0], wl.eos_id, wl.pad_id)
    it = iter(rows)
    for t in range(wl.T):
        bm.step(wl.logp(t)[0])
        for i in range(wl.k):
            r = next(it)
            assert [int(r[0]), int(r[1])] == [t, i]
            assert (int(r[2]), int(r[3])) == (int(bm.token[i]), int(bm.backptr[i]))
            assert r[4] == np.float32(bm.score[i]).tobytes().hex()
            assert (int(r[5]), int(r[6], 16)) == (int(bm.flags[i]), int(bm.met[i]))
