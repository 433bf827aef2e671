"""Pins for the oracle's variants of the experimental set-up: allocation without adjustment
(Sec. 5, the simulated GBS baseline), completed hypotheses stored with score/length (Sec. 4;
Fig. 9 caption), threshold pruning against the best completed hypothesis (Sec. 4, Sec. 6.3) and
the all-completed stopping test (Sec. 4).  CPU only."""
from __future__ import annotations

import itertools

import numpy as np
import pytest

import oracle
import synth_inputs as si
from oracle import brute


# ---- Sec. 5: the room of a bank does not change -------------------------------------------
def test_fixed_allocation_is_the_clipped_base_split():
    for k in range(1, 9):
        for C in range(0, 5):
            base, rem = divmod(k, C + 1)
            for cnt in itertools.product(range(0, 5), repeat=C + 1):
                a = oracle.allocate(k, cnt, adjust=False)
                for b in range(C + 1):
                    room = base + (rem if b == C else 0)
                    assert a[b] == min(room, cnt[b])
                assert a.sum() <= k
                # where every bank can fill its room, adjustment has nothing to move
                if all(cnt[b] >= base + (rem if b == C else 0) for b in range(C + 1)):
                    assert list(a) == list(oracle.allocate(k, cnt, adjust=True))
                # adjustment only ever fills more of the beam
                assert a.sum() <= oracle.allocate(k, cnt, adjust=True).sum()


def test_gbs_simulation_gives_every_bank_the_base_beam():
    """Sec. 5: beam b(C+1) and no adjustment = b slots for every bank, as in grid beam search."""
    for b, C in itertools.product((1, 5, 10), (0, 1, 3, 7)):
        k = b * (C + 1)
        cnt = [1000] * (C + 1)
        assert list(oracle.allocate(k, cnt, adjust=False)) == [b] * (C + 1)
        cnt[C // 2] = 2
        a = oracle.allocate(k, cnt, adjust=False)
        assert a[C // 2] == min(2, b) and all(a[x] == b for x in range(C + 1) if x != C // 2)


# ---- brute-force enumeration of the variants ------------------------------------------------
VARIANTS = [
    dict(adjust=False),
    dict(normalize=True),
    dict(prune=3.0),
    dict(prune=0.0, normalize=True),
    dict(adjust=False, normalize=True, prune=6.0),
]


def _oracle_kwargs(v):
    return dict(adjust=v.get("adjust", True), normalize_finished=v.get("normalize", False),
                prune_threshold=v.get("prune"))


@pytest.mark.parametrize("vi", range(len(VARIANTS)))
@pytest.mark.parametrize("seed", range(40))
def test_variants_match_brute_force(seed, vi):
    v = VARIANTS[vi]
    rs = si.Stream(seed, 177)
    k = rs.randint(2, 6)
    V = rs.randint(6, 40)
    T = rs.randint(5, 10)
    wl = si.make_small(500 + seed, 1, k, V, T, max_phrases=3, max_len=3, dup_prob=0.4)
    wl.eos_switch = 2
    wl.eos_high = 0.5
    phrases = wl.constraints[0]
    bm = oracle.SentenceBeam(k, V, phrases, wl.eos_id, wl.pad_id, **_oracle_kwargs(v))
    beam = [None] * k
    beam[0] = brute.Hyp(np.float32(0.0), [0] * len(phrases))
    for t in range(T):
        logp = wl.logp(t)[0]
        new, info = brute.step(beam, logp, phrases, wl.eos_id, wl.pad_id, **v)
        bm.step(logp, debug=True)
        assert list(bm.dbg["alloc"]) == info["alloc"]
        assert bm.all_finished == int(info["all_finished"])
        assert bm.any_finished == int(info["any_finished"])
        for i, item in enumerate(new):
            if item is None:
                assert bm.flags[i] == oracle.FLAG_DEAD and bm.backptr[i] == -1
                assert bm.token[i] == wl.pad_id and bm.score[i] == -np.inf and bm.len[i] == 0
                continue
            w, h, hyp = item
            assert (int(bm.token[i]), int(bm.backptr[i])) == (w, h)
            assert np.float32(bm.score[i]).tobytes() == np.float32(hyp.score).tobytes()
            assert int(bm.met[i]) == brute.met_mask(phrases, hyp)
            assert bool(bm.flags[i] & oracle.FLAG_FINISHED) == hyp.finished
            assert int(bm.len[i]) == hyp.length
        beam = [None if it is None else it[2] for it in new]


# ---- Sec. 4: score / number of words, for completed hypotheses only ---------------------------
def _path_sum(logps, hist_tok, hist_bp, t, slot, eos_id):
    """fp32 sum of the log-probs along the back-pointer path that ends in `slot` after step t,
    added in the order of generation, up to and including end-of-sentence."""
    path = []
    for u in range(t, -1, -1):
        parent = int(hist_bp[u][slot])
        path.append((u, parent, int(hist_tok[u][slot])))
        slot = parent
    s = np.float32(0.0)
    n = 0
    for u, parent, w in reversed(path):
        s = np.float32(s + logps[u][parent, w])
        n += 1
        if w == eos_id:
            break
    return s, n


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("normalize", [False, True])
def test_stored_score_is_the_path_sum_over_the_length(seed, normalize):
    k, V, T = 6, 50, 14
    wl = si.make_small(900 + seed, 1, k, V, T, max_phrases=2, max_len=2)
    wl.eos_switch = 3
    wl.eos_high = 0.0
    phrases = wl.constraints[0]
    bm = oracle.SentenceBeam(k, V, phrases, wl.eos_id, wl.pad_id, normalize_finished=normalize)
    logps, n_done = [], 0
    for t in range(T):
        logps.append(wl.logp(t)[0].copy())
        bm.step(logps[-1])
        for i in range(k):
            if bm.flags[i] == oracle.FLAG_DEAD:
                continue
            s, n = _path_sum(logps, bm.hist_token, bm.hist_backptr, t, i, wl.eos_id)
            assert n == bm.len[i]
            if (bm.flags[i] & oracle.FLAG_FINISHED) and normalize:
                assert bm.score[i] == np.float32(s) / np.float32(n)
                n_done += 1
            else:
                assert bm.score[i] == s
    if normalize:
        assert n_done > 0
        # the returned hypothesis is the completed one with the best stored score
        toks, ln, sc, status = bm.finalize(T)
        done = [i for i in range(k) if bm.flags[i] & oracle.FLAG_FINISHED]
        assert status == 1 and sc == max(bm.score[i] for i in done)
        first = min(i for i in done if bm.score[i] == sc)
        assert ln == bm.len[first] and toks[ln - 1] == wl.eos_id


# ---- Sec. 4 / Sec. 6.3: threshold pruning ---------------------------------------------------
def _clone(bm, **kw):
    c = oracle.SentenceBeam(bm.k, bm.V, bm.phrases, bm.eos_id, bm.pad_id, **kw)
    for name in ("score", "met", "ip", "iq", "flags", "len", "token", "backptr"):
        setattr(c, name, getattr(bm, name).copy())
    return c


@pytest.mark.parametrize("seed", range(16))
def test_pruned_step_is_the_unpruned_step_with_the_losers_struck_out(seed):
    k, V, T = 8, 60, 12
    theta = [0.0, 1.5, 4.0, 20.0][seed % 4]
    normalize = bool(seed & 4)
    wl = si.make_small(1300 + seed, 1, k, V, T, max_phrases=2, max_len=2)
    wl.eos_switch = 2
    wl.eos_high = -1.0
    bm = oracle.SentenceBeam(k, V, wl.constraints[0], wl.eos_id, wl.pad_id,
                             normalize_finished=normalize, prune_threshold=theta)
    n_pruned = 0
    for t in range(T):
        logp = wl.logp(t)[0]
        plain = _clone(bm, normalize_finished=normalize).step(logp)
        bm.step(logp)
        live = plain.flags != oracle.FLAG_DEAD
        done = live & ((plain.flags & oracle.FLAG_FINISHED) != 0)
        keep = live.copy()
        if done.any():
            best = plain.score[done].max()
            assert best in bm.score                                  # the best completed one stays
            keep &= ~(plain.score < np.float32(best - np.float32(theta)))
            # survivors are within the threshold of the best completed hypothesis
            assert (best.astype(np.float64) - plain.score[keep].astype(np.float64) <= theta + 1e-4).all()
        idx = np.flatnonzero(keep)
        n_pruned += int(live.sum()) - len(idx)
        for name in ("token", "backptr", "score", "flags", "met", "ip", "iq", "len"):
            got, want = getattr(bm, name), getattr(plain, name)
            assert got[:len(idx)].tobytes() == want[idx].tobytes(), (name, t)
        assert (bm.flags[len(idx):] == oracle.FLAG_DEAD).all() and (bm.score[len(idx):] == -np.inf).all()
        assert (bm.backptr[len(idx):] == -1).all() and (bm.token[len(idx):] == wl.pad_id).all()
        assert bm.all_finished == int(len(idx) > 0 and ((bm.flags[:len(idx)] & 1) == 1).all())
    if theta < 20.0:
        assert n_pruned > 0


def test_a_huge_threshold_prunes_nothing_and_a_finished_beam_stays_put():
    k, V, T = 5, 40, 16
    wl = si.make_small(77, 1, k, V, T, max_phrases=2, max_len=2)
    wl.eos_switch = 2
    wl.eos_high = 3.0
    a = oracle.SentenceBeam(k, V, wl.constraints[0], wl.eos_id, wl.pad_id)
    b = oracle.SentenceBeam(k, V, wl.constraints[0], wl.eos_id, wl.pad_id, prune_threshold=1e30)
    c = oracle.SentenceBeam(k, V, wl.constraints[0], wl.eos_id, wl.pad_id, normalize_finished=True,
                            prune_threshold=2.0)
    stopped_at = None
    for t in range(T):
        logp = wl.logp(t)[0]
        a.step(logp)
        b.step(logp)
        before = (c.score.copy(), c.len.copy(), c.met.copy())
        was_done = c.all_finished
        c.step(logp)
        for name in ("token", "backptr", "score", "flags", "met", "len"):
            assert getattr(a, name).tobytes() == getattr(b, name).tobytes()
        if was_done:
            # Sec. 4: decoding may stop here - further steps only carry the same hypotheses along
            # (now in the order of their stored scores)
            assert c.all_finished
            live = c.flags != oracle.FLAG_DEAD
            par = c.backptr[live]
            assert sorted(par.tolist()) == list(range(int(live.sum()))) and (c.token[live] == wl.pad_id).all()
            assert c.score[live].tobytes() == before[0][par].tobytes()
            assert c.len[live].tobytes() == before[1][par].tobytes()
            assert c.met[live].tobytes() == before[2][par].tobytes()
            assert (c.score[live][:-1] >= c.score[live][1:]).all()
        elif c.all_finished:
            stopped_at = t
    assert stopped_at is not None and stopped_at < T - 1


# ---- 16-bit log-probs: the exactness contract ------------------------------------------------
def _decode16(bits: int, ebits: int, mbits: int) -> float:
    """Value of a 16-bit binary float from its fields, in exact Python arithmetic."""
    sign = -1.0 if bits >> 15 else 1.0
    e = (bits >> mbits) & ((1 << ebits) - 1)
    m = bits & ((1 << mbits) - 1)
    bias = (1 << (ebits - 1)) - 1
    if e == (1 << ebits) - 1:
        return sign * float("inf") if m == 0 else float("nan")
    if e == 0:
        return sign * m * 2.0 ** (1 - bias - mbits)
    return sign * (1.0 + m * 2.0 ** -mbits) * 2.0 ** (e - bias)


@pytest.mark.parametrize("fmt,ebits,mbits", [("f16", 5, 10), ("bf16", 8, 7)])
def test_widening_is_exact_for_every_bit_pattern(fmt, ebits, mbits):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    with np.errstate(invalid="ignore"):
        got = oracle.widen16(bits, fmt)
    want = np.array([_decode16(int(b), ebits, mbits) for b in bits], dtype=np.float64)
    with np.errstate(invalid="ignore"):
        ok = (got.astype(np.float64) == want) | (np.isnan(got) & np.isnan(want))
    assert ok.all()
    assert (np.signbit(got) == (bits >> 15).astype(bool)).all()         # -0.0 stays -0.0


@pytest.mark.parametrize("fmt,ebits,mbits", [("f16", 5, 10), ("bf16", 8, 7)])
def test_narrowing_rounds_to_the_nearest_value_ties_to_even(fmt, ebits, mbits):
    """The input generator's rounding: the nearest representable value, checked against all
    neighbours on a sample that includes exact ties."""
    with np.errstate(invalid="ignore"):
        grid = oracle.widen16(np.arange(65536, dtype=np.uint32).astype(np.uint16), fmt).astype(np.float64)
    finite = np.isfinite(grid)
    vals = np.sort(np.unique(grid[finite]))
    rs = np.random.default_rng(7)
    x = np.concatenate([-np.exp(rs.uniform(-12, 4, 4000)), (vals[1000:1200] + vals[1001:1201]) / 2,
                        [0.0, -0.0, -np.inf]]).astype(np.float32)
    got = oracle.widen16(si.narrow16(x, fmt), fmt).astype(np.float64)
    for xi, gi in zip(x.astype(np.float64), got):
        if not np.isfinite(xi):
            assert gi == xi
            continue
        j = np.searchsorted(vals, xi)
        near = vals[max(0, j - 1):j + 2]
        best = np.abs(near - xi).min()
        assert abs(gi - xi) == best, (xi, gi)
        ties = near[np.abs(near - xi) == best]
        if len(ties) == 2:                       # exact tie: the one with an even last bit
            b = int(si.narrow16(np.array([xi], np.float32), fmt)[0])
            assert b & 1 == 0


# ---- Sec. 3.3: the best completed hypothesis, also when it has left the beam ---------------------
def _walk_completed(scores, flags, lens, normalize):
    """Every completed hypothesis on every recorded beam: (value per word, step, slot)."""
    seen = []
    for t in range(len(scores)):
        for h in range(len(scores[t])):
            if flags[t][h] == oracle.FLAG_DEAD or not (flags[t][h] & oracle.FLAG_FINISHED):
                continue
            q = np.float32(scores[t][h]) if normalize else np.float32(scores[t][h]) / np.float32(lens[t][h])
            seen.append((q, t, h))
    return seen


def test_tracked_finalize_hand_worked_drop_out():
    """k = 2, no constraints, ids: 0 pad, 2 end-of-sentence.  Step 0: the beam becomes [3 (-0.1),
    end-of-sentence (-3.0, completed, one word)].  Step 1: both continuations of 3 (-0.6, -1.1) beat
    the completed hypothesis, which leaves the beam.  Step 2: one of them completes at -10.6 over
    three words = -3.53 per word, worse than -3.0 per word.  The bare reading returns the three-word
    hypothesis (the only completed one on the last beam); the tracking variant returns the one-word
    hypothesis seen at step 0."""
    V, k, T, lo = 6, 2, 3, np.float32(-50.0)
    lp = np.full((T, k, V), lo, np.float32)
    lp[0, 0, 3], lp[0, 0, 2] = -0.1, -3.0
    lp[1, 0, 4], lp[1, 0, 5] = -0.5, -1.0
    lp[2, 0, 2], lp[2, 0, 3] = -10.0, -20.0
    lp[2, 1, 3] = -0.3
    res = {}
    for track in (False, True):
        bm = oracle.SentenceBeam(k, V, [], 2, 0, track_completed=track)
        for t in range(T):
            bm.step(lp[t])
            if t == 0:
                assert list(bm.token) == [3, 2] and list(bm.flags) == [0, 1]
            if t == 1:
                assert list(bm.token) == [4, 5] and list(bm.flags) == [0, 0]
        assert list(bm.token) == [3, 2] and list(bm.backptr) == [1, 0] and list(bm.flags) == [0, 1]
        res[track] = bm.finalize(4)
    toks, ln, sc, status = res[False]
    assert status == 1 and ln == 3 and list(toks) == [3, 4, 2, 0] and sc == np.float32(np.float32(-0.1) + np.float32(-0.5)) + np.float32(-10.0)
    toks, ln, sc, status = res[True]
    assert status == 1 and ln == 1 and list(toks) == [2, 0, 0, 0] and sc == np.float32(-3.0)


def test_tracked_finalize_returns_the_best_completed_hypothesis_ever_seen():
    """The variant that remembers completed hypotheses, on decodes in which completed hypotheses
    get onto the beam and are pushed off again: what the end of decoding returns scores at least as
    well, per word, as every completed hypothesis that sat on any beam (walked here from the recorded
    beams; its value recomputed from the log-probs along its back-pointers), its tokens are the
    back-trace from where it was first seen, and where it is still on the last beam, alone with its
    value, the bare reading returns the same."""
    dropped = agree = 0
    for seed in range(400):
        normalize = bool(seed & 1)
        k, V, T = [2, 3, 4, 5][seed % 4], 8, 12
        cons = [[], [[5]], [[4, 6]], [[3], [7]]][(seed // 4) % 4]
        eos, pad = 2, 0
        bm = oracle.SentenceBeam(k, V, cons, eos, pad, track_completed=True, normalize_finished=normalize)
        plain = oracle.SentenceBeam(k, V, cons, eos, pad, normalize_finished=normalize)
        logps, scores, flags, lens = [], [], [], []
        for t in range(T):
            logps.append(si.two_profile_logp(700 + seed, t, 1, k, V)[0])
            bm.step(logps[-1])
            plain.step(logps[-1])
            assert bm.score.tobytes() == plain.score.tobytes() and bm.token.tobytes() == plain.token.tobytes()
            scores.append(bm.score.copy())
            flags.append(bm.flags.copy())
            lens.append(bm.len.copy())
        toks, ln, sc, status = bm.finalize(T)
        p_toks, p_ln, p_sc, p_status = plain.finalize(T)
        seen = _walk_completed(scores, flags, lens, normalize)
        if not seen:
            assert status == 0 and p_status == 0
            assert toks.tobytes() == p_toks.tobytes() and (ln, sc) == (p_ln, p_sc)
            continue
        best_q = max(q for q, _, _ in seen)
        t0, h0 = min((t, h) for q, t, h in seen if q == best_q)
        assert status == 1 and ln == lens[t0][h0] and sc == scores[t0][h0]
        # its tokens: back-pointers from (t0, h0); its value: the log-probs along that path
        want, slot = [], h0
        for u in range(t0, -1, -1):
            want.append(int(bm.hist_token[u][slot]))
            slot = int(bm.hist_backptr[u][slot])
        want = want[::-1][:ln]
        assert list(toks[:ln]) == want and want[-1] == eos and (toks[ln:] == pad).all()
        s, n = _path_sum(logps, bm.hist_token, bm.hist_backptr, t0, h0, eos)
        assert n == ln and best_q == np.float32(s) / np.float32(n)
        last_vals = [q for q, _, _ in _walk_completed([scores[-1]], [flags[-1]], [lens[-1]], normalize)]
        if best_q not in last_vals:
            # it has left the beam: the bare reading returns something worse per word, or nothing
            dropped += 1
            assert p_status == 0 or (p_sc if normalize else np.float32(p_sc) / np.float32(p_ln)) < best_q
        elif last_vals.count(best_q) == 1 and len({(t, h) for q, t, h in seen if q == best_q and t == t0}) == 1:
            assert p_status == 1 and (p_ln, p_sc) == (ln, sc) and p_toks.tobytes() == toks.tobytes()
            agree += 1
    assert dropped >= 10 and agree >= 100, (dropped, agree)
