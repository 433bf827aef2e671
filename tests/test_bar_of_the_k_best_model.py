"""The argument behind the merge phase's shortcut for the sentence's k best (Sec. 3.1 item 1), as a
host model checked against brute force.

The device code never sorts the sentence's k best keys.  It merges the 32-bit score images of the
row lists (top 64 kept at every merge, lists whose head is below place k-1 of the running chain
skipped, the greatest dropped image remembered), reads the k-th best score, and decides:
  * exactly k listed keys have that score or a better one (and, at k = 64 where every place is taken,
    nothing as good was dropped): those k keys are the k best;
  * otherwise the same merge over the low words of the keys with exactly that score finds the last
    one that gets in.
This file restates those steps on plain Python lists and checks the outcome - which keys are among
the k best - against a full sort of all keys, on inputs full of ties, with rows longer than their
64-entry lists, for every beam size class the kernel is laid out for.  No GPU, no library call: it
pins the reasoning, the GPU tests pin the code.
"""
import random

import pytest

WAVES = 4
KEEP = 64


def merge_keep(a, b, fell):
    """Top KEEP of two decreasing lists (equal values allowed); fell[0] = greatest value dropped."""
    allv = sorted(a + b, reverse=True)
    for v in allv[KEEP:]:
        fell[0] = max(fell[0], v)
    return allv[:KEEP]


def place(lst, i):
    return lst[i] if i < len(lst) else 0


def wave_best(lists, kth, look, fell):
    """Two chains side by side (rows 0, 2, 4, .. and 1, 3, 5, .. of the wave), joined at the end."""
    a0 = list(lists[0]) if lists else []
    a1 = list(lists[1]) if len(lists) > 1 else []
    for i in range(2, len(lists), 2):
        s0 = lists[i]
        s1 = lists[i + 1] if i + 1 < len(lists) else []
        n0, n1 = True, i + 1 < len(lists)
        if look:
            n0 = bool(s0) and s0[0] >= place(a0, kth)
            n1 = bool(s1) and s1[0] >= place(a1, kth)
        if n0:
            a0 = merge_keep(a0, s0, fell)
        if n1:
            a1 = merge_keep(a1, s1, fell)
    return merge_keep(a0, a1, fell) if a1 else a0


def block_best(per_wave, fell):
    x = merge_keep(per_wave[0], per_wave[1], fell)
    y = merge_keep(per_wave[2], per_wave[3], fell)
    return merge_keep(x, y, fell)


def members_by_model(rows, k):
    """rows[h] = decreasing list of distinct keys (score, low) with at most KEEP entries.  Returns the
    set of keys the model puts among the k best."""
    look = k > 32                                  # sixteen rows a wave: lists are looked at first
    by_wave = [[rows[h] for h in range(w, len(rows), WAVES)] for w in range(WAVES)]
    fell = [0]
    scores = [wave_best([[s for s, _ in r] for r in rs], k - 1, look, fell) for rs in by_wave]
    accs = block_best(scores, fell)
    tau_s = place(accs, k - 1)
    if tau_s == 0:                                 # fewer than k keys in all: every key is in
        return {key for r in rows for key in r}
    settled = sum(1 for v in accs if v >= tau_s) == k
    if settled and k == KEEP:
        settled = fell[0] < tau_s
    if settled:
        return {key for r in rows for key in r if key[0] >= tau_s}
    need = k - sum(1 for v in accs if v > tau_s)
    unused = [0]
    lows = [wave_best([[lo for s, lo in r if s == tau_s] for r in rs], need - 1, True, unused) for rs in by_wave]
    accl = block_best(lows, unused)
    tau_l = accl[need - 1]
    return {key for r in rows for key in r if key[0] > tau_s or (key[0] == tau_s and key[1] >= tau_l)}


def random_rows(rng, k, levels, row_len):
    """k rows of row_len distinct keys each; scores on a few levels (ties everywhere), low words
    distinct over the whole sentence.  Each row keeps its best KEEP keys, as the stream phase does."""
    lows = rng.sample(range(1, 1 << 20), k * row_len)
    rows = []
    for h in range(k):
        n = rng.choice([0, 1, 3, row_len // 2, row_len]) if rng.random() < 0.3 else row_len
        keys = [(rng.randint(1, levels) + (rng.randint(0, 3) if rng.random() < 0.2 else 0), lows[h * row_len + j])
                for j in range(n)]
        rows.append(sorted(keys, reverse=True)[:KEEP])
    return rows


@pytest.mark.parametrize("k", [1, 2, 3, 5, 12, 16, 20, 31, 32, 33, 48, 63, 64])
@pytest.mark.parametrize("levels", [1, 2, 5, 40, 100000])
def test_the_model_finds_exactly_the_k_best(k, levels):
    rng = random.Random(1000 * k + levels)
    for trial in range(60):
        rows = random_rows(rng, k, levels, rng.choice([4, 20, 64, 100]))
        every = sorted((key for r in rows for key in r), reverse=True)
        want = set(every[:k])
        got = members_by_model(rows, k)
        assert got == want, (k, levels, trial, len(every))


def test_a_tie_hidden_among_dropped_keys_is_noticed():
    """k = 64, two rows of 64 keys, all with one score: every place of the merged list is taken and
    counting alone cannot see the tie; the greatest dropped image gives it away."""
    rows = [[(7, 1000 - j) for j in range(64)], [(7, 2000 - j) for j in range(64)]] + [[] for _ in range(62)]
    every = sorted((key for r in rows for key in r), reverse=True)
    assert members_by_model(rows, 64) == set(every[:64])


def test_a_list_whose_head_ties_with_the_running_bar_is_not_skipped():
    """k = 40: one row fills all k places with one score, a later row of the same chain holds one more
    key with that score.  Skipping it (its head does not beat place k-1) would leave exactly k keys in
    sight and let the k+1 keys with that score all pass."""
    k = 40
    rows = [[] for _ in range(k)]
    rows[0] = [(9, 5000 - j) for j in range(40)]
    rows[8] = [(9, 9000)]                          # wave 0 again, the chain row 0 is in; best low word of all
    every = sorted((key for r in rows for key in r), reverse=True)
    got = members_by_model(rows, k)
    assert got == set(every[:k])
    assert (9, 9000) in got and (9, 5000 - 39) not in got
