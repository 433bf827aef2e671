"""-m gpu: the HIP path, called through the C ABI, against the CPU oracle."""
import itertools
import os

import numpy as np
import pytest

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu


def _harness():
    import harness                      # needs torch + a GPU
    return harness


@pytest.fixture(scope="module")
def torch_gpu():
    import torch
    assert torch.cuda.is_available()
    return torch


def test_allocation_device_matches_oracle(torch_gpu):
    """Sec. 3.2 on one wavefront vs the oracle: exhaustive small cases, the figure cases,
    random large ones incl. 64 constraint tokens and k < C."""
    import paper_1804_06609_amd as dba
    cases = []
    for k in range(1, 7):
        for C in range(0, 4):
            for cnt in itertools.product(range(0, k + 2), repeat=C + 1):
                cases.append((k, C, list(cnt)))
    rs = si.Stream(4242, 1)
    for _ in range(6000):
        k = rs.randint(1, 64)
        C = rs.randint(0, 64)
        style = rs.randint(0, 3)
        cnt = []
        for b in range(C + 1):
            if style == 0:
                cnt.append(rs.randint(0, 3))
            elif style == 1:
                cnt.append(rs.randint(0, 40) if rs.randint(0, 4) == 0 else 0)
            elif style == 2:
                cnt.append(rs.randint(0, 2 * k))
            else:
                cnt.append(0 if b > rs.randint(0, C) else rs.randint(0, 9))
        cases.append((k, C, cnt))
    n = len(cases)
    kk = np.array([c[0] for c in cases], np.int32)
    CC = np.array([c[1] for c in cases], np.int32)
    cnt = np.zeros((n, 65), np.int32)
    for i, c in enumerate(cases):
        cnt[i, :len(c[2])] = c[2]
    scratch = torch_gpu.empty(n * 132 * 4, dtype=torch_gpu.uint8, device="cuda")
    for adjust in (True, False):         # Sec. 3.2, and the fixed split of Sec. 5
        alloc = np.full((n, 65), -7, np.int32)
        dba.dba_debug_allocate(kk, CC, cnt, alloc, scratch.data_ptr(), scratch.numel(),
                               torch_gpu.cuda.current_stream().cuda_stream, adjust=adjust)
        for i, (k, C, c) in enumerate(cases):
            want = oracle.allocate(k, c, adjust=adjust)
            assert list(alloc[i, :C + 1]) == list(want), (adjust, k, C, c, alloc[i, :C + 1], want)
            assert (alloc[i, C + 1:] == 0).all()


def test_wave_selection_primitives(torch_gpu):
    """The 64-lane sort / merge / insert networks (DPP and permlane exchanges) against a host
    sort, on random distinct keys, keys differing only in the low word, and sentinels; the 32-bit
    merge on the keys' high words (all equal in every fourth case)."""
    import paper_1804_06609_amd as dba
    n = 512
    rng = np.random.default_rng(7)
    keys = rng.integers(1, 2 ** 63, size=(n, 128), dtype=np.int64).astype(np.uint64)
    keys[1::4] = (keys[1::4] & np.uint64(0xFFFF)) | (np.uint64(0x3F800000) << np.uint64(32)) | \
        (np.arange(128, dtype=np.uint64)[None, :] << np.uint64(16))      # equal high words
    keys[2::4, 40:64] = 0                                                  # short first list
    keys[2::4, 100:] = 0                                                   # short second list
    keys[3::4, :64] = 0                                                    # empty first list
    vals = rng.standard_normal((n, 64)).astype(np.float32) * 10
    vals[5::8, 10:30] = -np.inf
    vals[6::8, :] = np.float32(-3.25)
    out = np.zeros((n, 256), np.uint64)
    fout = np.zeros((n, 64), np.float32)
    scratch = torch_gpu.empty(n * 3584, dtype=torch_gpu.uint8, device="cuda")
    dba.dba_debug_wave_select(keys, vals, out, fout, scratch.data_ptr(), scratch.numel(),
                              torch_gpu.cuda.current_stream().cuda_stream)
    for i in range(n):
        a = np.sort(keys[i, :64])[::-1]
        assert (out[i, :64] == a).all(), i
        both = np.sort(keys[i])[::-1][:64]
        assert (out[i, 64:128] == both).all(), i
        ins = np.sort(np.concatenate([keys[i, :64], keys[i, 64:72][keys[i, 64:72] != 0]]))[::-1][:64]
        if (keys[i, 64:72] != 0).all():
            assert (out[i, 128:192] == ins).all(), i
        assert fout[i].tobytes() == np.sort(vals[i])[::-1].tobytes(), i
        hi = np.sort(keys[i] >> np.uint64(32))[::-1]
        assert ((out[i, 192:] & np.uint64(0xFFFFFFFF)) == hi[:64]).all(), i
        assert ((out[i, 192:] >> np.uint64(32)) == hi[64]).all(), i


@pytest.mark.parametrize("seed", range(24))
def test_small_fuzz(torch_gpu, seed):
    """Odd small shapes: k=1, V not a multiple of 4 (unaligned rows), repeated tokens,
    sentences without constraints, boosted constraint tokens, early EOS."""
    rs = si.Stream(seed, 5)
    B = rs.randint(1, 5)
    k = [1, 2, 3, 5, 8, 13, 33, 64][seed % 8]
    V = max(k + 3, [37, 64, 130, 257, 1001, 1023, 2050, 4099][(seed // 3) % 8])
    T = rs.randint(6, 14)
    wl = si.make_small(9000 + seed, B, k, V, T, max_phrases=5, max_len=4, dup_prob=0.35)
    wl.eos_switch = T // 2
    _harness().run_parity(wl)


def test_many_constraints_small_beam(torch_gpu):
    """C >= k (Sec. 5): 64 single-token and phrasal constraints, k=3."""
    B, k, V, T = 3, 3, 3000, 40
    cons = si.fixed_total_constraints(31, B, V, 64, max_len=3)
    wl = si.Workload(B=B, k=k, V=V, T=T, seed=31, constraints=cons,
                     boost_tokens=[[w for p in s for w in p] for s in cons], boost_prob=0.2)
    _harness().run_parity(wl)


def test_tiny_shapes(torch_gpu):
    """The smallest shapes: V from 5 up (ids 0..3 are reserved by the generator), k from 1 to V, one
    and three steps, with and without constraints."""
    h = _harness()
    n = 0
    for V in (5, 6, 7, 9, 16):
        for k in sorted({1, 2, V // 2, V - 1, V}):
            for T in (1, 3):
                wl = si.make_small(7000 + 31 * V + k, 2, k, V, T, max_phrases=2, max_len=2, dup_prob=0.5)
                wl.eos_switch = 1
                h.run_parity(wl)
                n += 1
    assert n >= 40


class _TieHeavy(si.Workload):
    """Log-probs on a few levels only: almost every element ties with thousands of others, so the
    order is decided by coordinates everywhere and far more elements than usual reach the
    thresholds (the stages of the stream phase fill up and are folded many times per row)."""

    levels = 3

    def logp(self, t, sentences=None, out=None):
        lp = super().logp(t, sentences, out)
        q = np.round(lp * (self.levels / 8.0)) * (8.0 / self.levels)
        q[..., self.eos_id] = lp[..., self.eos_id]
        lp[...] = q.astype(np.float32)
        return lp


@pytest.mark.parametrize("levels,fmt,k", [(3, None, 12), (1, None, 12), (6, "bf16", 12), (2, "f16", 12),
                                          (2, None, 64), (5, "bf16", 64), (3, None, 33), (1, None, 4)])
def test_ties_everywhere(torch_gpu, levels, fmt, k):
    """Also the beam sizes at which the last places of the k best are contested among keys that
    the 32-bit merges of the merge phase cannot tell apart (k = 64: every place of the lists is
    taken, the tie shows only in what was dropped)."""
    base = si.make_small(5151 + levels, 3, k, 6007, 9, max_phrases=4, max_len=3, dup_prob=0.3)
    wl = _TieHeavy(B=base.B, k=base.k, V=base.V, T=base.T, seed=base.seed, constraints=base.constraints,
                   boost_tokens=base.boost_tokens, boost_value=4.0, boost_prob=0.35)
    wl.levels = levels
    wl.eos_switch = 5
    _harness().run_parity(wl, logp_format=fmt)


@pytest.mark.parametrize("seed", range(16))
def test_ties_fuzz(torch_gpu, seed):
    """Tie-heavy decodes over beam sizes, vocabularies and tie densities: the last places of the
    k best, the rows' bests and the constraint tokens are all contested by equal sums."""
    rs = si.Stream(seed, 77)
    k = [2, 5, 20, 48, 64, 63, 16, 32][seed % 8]
    V = [300, 2000, 900, 4100][(seed // 2) % 4]
    base = si.make_small(8800 + seed, 2, k, V, 6, max_phrases=5, max_len=3, dup_prob=0.3)
    wl = _TieHeavy(B=base.B, k=base.k, V=base.V, T=base.T, seed=base.seed, constraints=base.constraints,
                   boost_tokens=base.boost_tokens, boost_value=float(rs.randint(0, 3)) * 8.0 / 3.0,
                   boost_prob=0.5)
    wl.levels = [1, 2, 3, 4, 8, 16][rs.randint(0, 5)]
    wl.eos_switch = 3
    import paper_1804_06609_amd as dba
    # the second half of the seeds with four waves a sentence in the merge phase whatever the beam size
    _harness().run_parity(wl, logp_format=[None, None, "bf16", "f16"][rs.randint(0, 3)],
                          options={dba.DBA_OPT_MERGE_WAVES: 0 if seed < 8 else 4})


class _ContestedLastPlaces(si.Workload):
    """Step 0 gives all k hypotheses one score; at step 1 hypothesis 0 has k tokens at one level and
    hypothesis 8 - same wave, same chain of merges in the merge phase - a single token at that level:
    k+1 sums tie for the k places, and the list of hypothesis 8 has a head that only equals, never
    beats, the k-th best found before it.  Later steps are the generator's."""

    def logp(self, t, sentences=None, out=None):
        lp = super().logp(t, sentences, out)
        if t == 0:
            lp[...] = np.float32(-2.0)
            lp[..., self.eos_id] = np.float32(-60.0)
        elif t == 1:
            lp[...] = np.float32(-30.0)
            lp[:, 0, 100:100 + self.k] = np.float32(-1.0)
            lp[:, 8, 7] = np.float32(-1.0)
            lp[:, 3, 50:60] = np.float32(-1.5)
        return lp


@pytest.mark.parametrize("k", [40, 64, 20])
def test_contested_last_places(torch_gpu, k):
    wl = _ContestedLastPlaces(B=2, k=k, V=3000, T=4, seed=77, constraints=[[], [[9, 10], [700]]])
    wl.eos_switch = 1 << 30
    _harness().run_parity(wl)


class _TiedConstraintToken(si.Workload):
    """k = 64.  At step 1 hypothesis 0 has 65 tokens at one level: 64 ordinary ones with the lowest ids,
    which are the sentence's k best and fill the row's list, and the constraint token 500, which has the
    k-th best score too but is not among the k best nor in the list - it has to come in as a constraint
    candidate all the same (Sec. 3.1 item 2)."""

    def logp(self, t, sentences=None, out=None):
        lp = super().logp(t, sentences, out)
        if t == 0:
            lp[...] = np.float32(-2.0)
            lp[..., self.eos_id] = np.float32(-60.0)
        elif t == 1:
            lp[...] = np.float32(-30.0)
            lp[:, 0, 100:164] = np.float32(-1.0)
            lp[:, 0, 500] = np.float32(-1.0)
        return lp


def test_constraint_token_tied_with_the_k_best_but_not_one_of_them(torch_gpu):
    wl = _TiedConstraintToken(B=2, k=64, V=3000, T=4, seed=78, constraints=[[[500]], [[500, 9], [700]]])
    wl.eos_switch = 1 << 30
    _harness().run_parity(wl)
    ob = oracle.BatchBeam(wl.k, wl.V, wl.constraints, wl.eos_id, wl.pad_id)
    for t in range(2):
        ob.step(wl.logp(t))
    assert 500 in ob.stacked("token")[0].tolist()      # the case is what it claims to be


class _Masked(si.Workload):
    """A decoder with a restricted vocabulary: all but a few entries of every row are -inf (a
    different few in every row and step), so a sentence can have fewer than k finite sums, beams
    run partly empty, and constraint tokens are often impossible."""

    keep = 6

    def logp(self, t, sentences=None, out=None):
        lp = super().logp(t, sentences, out)
        n = lp.shape[0] * lp.shape[1]
        flat = lp.reshape(n, self.V)
        for r in range(n):
            rs = si.Stream(self.seed + 977 * t, r)
            allowed = {rs.randint(0, self.V - 1) for _ in range(rs.randint(1, self.keep))}
            allowed.add(self.eos_id if rs.randint(0, 2) == 0 else rs.randint(4, self.V - 1))
            if rs.randint(0, 1):
                allowed.update(w for p in self.constraints[(r // self.k) % len(self.constraints)] for w in p[:1])
            mask = np.ones(self.V, bool)
            mask[list(allowed)] = False
            flat[r, mask] = -np.inf
        return lp


@pytest.mark.parametrize("keep,fmt", [(2, None), (6, None), (12, "bf16"), (4, "f16")])
def test_restricted_vocabulary(torch_gpu, keep, fmt):
    base = si.make_small(6161 + keep, 4, 9, 1501, 10, max_phrases=3, max_len=2, dup_prob=0.2)
    wl = _Masked(B=base.B, k=base.k, V=base.V, T=base.T, seed=base.seed, constraints=base.constraints,
                 boost_tokens=base.boost_tokens, boost_value=4.0, boost_prob=0.35)
    wl.keep = keep
    wl.eos_switch = 4
    _harness().run_parity(wl, logp_format=fmt)


def test_many_sentences_long_decode(torch_gpu):
    """300 sentences (more workgroups in the merge phase than compute units), 150 steps of history,
    the set-up of Sec. 4 (per-word scores, pruning at 20), end-of-sentence likely from step 40 on."""
    wl = si.make_small(4242, 300, 7, 257, 150, max_phrases=4, max_len=3, dup_prob=0.3)
    wl.eos_switch = 40
    wl.eos_high = -2.0
    _harness().run_parity(wl, check_state_every=10, normalize=True, prune=20.0)


def test_most_candidates(torch_gpu):
    """The widest beam with 64 one-token constraints: k * (64 + 2) candidates per sentence at most,
    the largest candidate buffer the merge phase can need."""
    B, k, V, T = 2, 64, 5000, 5
    cons = si.fixed_total_constraints(61, B, V, 64, max_len=1)
    wl = si.Workload(B=B, k=k, V=V, T=T, seed=61, constraints=cons,
                     boost_tokens=[[w for p in s for w in p] for s in cons], boost_prob=0.5, boost_value=6.0)
    _harness().run_parity(wl)


@pytest.mark.parametrize("k,fmt", [(8, None), (33, None), (13, "bf16")])
def test_first_tokens_that_share_a_table_bucket(torch_gpu, k, fmt):
    """The device looks a token's phrases up in a table bucketed by the low six bits of the first token.
    Here phrases of one sentence begin with tokens that agree in those bits (70, 134, 198, 262), some
    begin with the very same token, some tokens of that bucket begin no phrase (326), and all of them are
    boosted so that they sit among the rows' best sums: the banks worked out at the end of a row and the
    state transition of the winners must take the one-by-one path through the bucket."""
    B, V, T = 4, 600, 14
    cons = [
        [[70, 5], [134], [198, 9, 10], [70, 6], [262, 134]],
        [[134, 70], [198], [134, 70, 11]],
        [[262], [70], [326 + 64, 70]],
        [[70, 134, 198], [134, 198], [198]],
    ]
    wl = si.Workload(B=B, k=k, V=V, T=T, seed=4300 + k, constraints=cons,
                     boost_tokens=[[70, 134, 198, 262, 326, 390] for _ in range(B)], boost_prob=0.6, boost_value=7.0)
    wl.eos_switch = 9
    _harness().run_parity(wl, logp_format=fmt)


def test_batch_equals_single_sentences(torch_gpu):
    """Sentences never interact: a batch run equals one-sentence runs of the same rows."""
    h = _harness()
    wl = si.make_config(3, T=12, B=4)
    wl.V = 5000
    wl.constraints = [[[4 + (w % (wl.V - 4)) for w in ph] for ph in s] for s in wl.constraints]
    wl.boost_tokens = [[4 + (w % (wl.V - 4)) for w in s] for s in wl.boost_tokens]
    fin = h.run_parity(wl)
    assert fin[0].shape == (4, 12)


VARIANTS = [
    dict(adjust=False),
    dict(normalize=True),
    dict(prune=3.0),
    dict(normalize=True, prune=20.0),          # the set-up of Sec. 4
    dict(adjust=False, normalize=True, prune=0.0),
]


@pytest.mark.parametrize("vi", range(len(VARIANTS)))
@pytest.mark.parametrize("seed", range(6))
def test_variants_small(torch_gpu, seed, vi):
    """Sec. 5 (no adjustment), Sec. 4 (completed hypotheses hold score/length; threshold pruning;
    the stopping test) on small odd shapes in which hypotheses complete early."""
    rs = si.Stream(seed, 6)
    B = rs.randint(1, 5)
    k = [2, 5, 13, 20, 33, 64][seed % 6]
    V = max(k + 3, [64, 257, 1001, 1023, 2050, 4099][(seed // 2) % 6])
    T = rs.randint(8, 14)
    wl = si.make_small(9300 + 10 * vi + seed, B, k, V, T, max_phrases=4, max_len=3, dup_prob=0.35)
    wl.eos_switch = 3
    wl.eos_high = [0.5, 3.0][seed % 2]
    _harness().run_parity(wl, **VARIANTS[vi])


@pytest.mark.parametrize("block", range(6))
def test_option_combinations_fuzz(torch_gpu, block):
    """Sixty small decodes in which everything varies at once: shape (k = 1..64, V = 37..9001), phrase
    count and length, repeated tokens, when end-of-sentence becomes likely, the element type of the
    log-probs, and every combination of the options (adjustment, per-word scores, pruning threshold,
    record of completed hypotheses), and the waves of the merge phase's workgroups."""
    for seed in range(10 * block, 10 * block + 10):
        rs = si.Stream(seed, 77)
        B = rs.randint(1, 6)
        k = [1, 2, 3, 5, 8, 13, 20, 33, 64][seed % 9]
        V = max(k + 3, [37, 64, 130, 257, 700, 1001, 1023, 2050, 4099, 9001][(seed // 3) % 10])
        T = rs.randint(6, 16)
        wl = si.make_small(20000 + seed, B, k, V, T, max_phrases=rs.randint(1, 8), max_len=rs.randint(1, 5),
                           dup_prob=[0.0, 0.35, 0.7][seed % 3])
        wl.eos_switch = rs.randint(2, T)
        wl.eos_high = [0.5, 2.0, 3.0][seed % 3]
        import paper_1804_06609_amd as dba
        _harness().run_parity(wl, adjust=bool(seed & 1), normalize=bool(seed & 2),
                              prune=[None, 20.0, 2.0, 0.0][(seed >> 2) & 3], track=bool(seed & 16),
                              logp_format=[None, None, "bf16", "f16"][(seed // 2) % 4],
                              options={dba.DBA_OPT_MERGE_WAVES: [0, 4, 8][(seed // 5) % 3]})


@pytest.mark.parametrize("waves", [4, 8])
@pytest.mark.parametrize("cfg,T,B", [(2, 20, None), (4, 30, 12), (5, 14, 3)])
def test_merge_phase_with_four_and_with_eight_waves(torch_gpu, cfg, T, B, waves):
    """DBA_OPT_MERGE_WAVES changes how a sentence's beam rows are dealt out to the waves of its
    workgroup in the second launch, never the result: k = 10, 20 and 64 (configs 2, 4 and 5, a few
    sentences, the first steps - where the candidates are most) with both fixed settings."""
    import paper_1804_06609_amd as dba
    wl = si.make_config(cfg, T=T) if B is None else si.make_config(cfg, T=T, B=B)
    _harness().run_parity(wl, options={dba.DBA_OPT_MERGE_WAVES: waves})


def test_paper_setup_config2(torch_gpu):
    """Config 2 shapes with the decoding set-up of Sec. 4: score per word for completed
    hypotheses, pruning threshold 20; end-of-sentence becomes likely after a third of the run."""
    wl = si.make_config(2, T=30)
    wl.eos_switch = 10
    _harness().run_parity(wl, normalize=True, prune=20.0)


@pytest.mark.parametrize("fmt", [None, "bf16"])
def test_paper_setup_config4(torch_gpu, fmt):
    """The headline shape (64 sentences, k = 20, V = 32000, 32 constraint tokens) with the decoding
    set-up of Sec. 4 - score per word for completed hypotheses, pruning threshold 20 - and
    end-of-sentence likely from step 12 on, so that hypotheses complete, beams shrink and the
    stopping test fires at full width; once on fp32 and once on bfloat16 log-probs."""
    wl = si.make_config(4, T=30)
    wl.eos_switch = 12
    _harness().run_parity(wl, normalize=True, prune=20.0, check_state_every=3, logp_format=fmt,
                          progress="config4/Sec.4")


def test_paper_setup_config5(torch_gpu):
    """The largest shape (B=128, k=64, V=50000) with the set-up of Sec. 4 and without the adjustment
    of Sec. 3.2 for a change; end-of-sentence likely from step 5 on.  The oracle follows all 128
    sentences through the 12 steps."""
    wl = si.make_config(5, T=12)
    wl.eos_switch = 5
    _harness().run_parity(wl, normalize=True, prune=20.0, adjust=False, check_state_every=3,
                          progress="config5/Sec.4")


@pytest.mark.parametrize("normalize,prune", [(False, None), (True, None), (False, 20.0), (True, 3.0)])
def test_completed_hypotheses_that_leave_the_beam(torch_gpu, normalize, prune):
    """Sec. 3.3 with the record of the best completed hypothesis: 240 short decodes (k = 2..5, with and
    without constraints) whose log-probs push completed hypotheses off the beam again; the end of
    decoding must return what the oracle's record returns - and, without per-word scores on the beam,
    something other than the bare reading for some sentences (the case the record exists for)."""
    B, V, T = 240, 8, 12
    shapes = [[], [[5]], [[4, 6]], [[3], [7]]]
    fins = {}
    for k in (2, 3, 4, 5):
        cons = [shapes[(b // 3) % 4] for b in range(B)]
        wl = si.TwoProfileWorkload(B=B, k=k, V=V, T=T, seed=8100 + k, constraints=cons)
        wl.eos_switch = 0
        for track in (True, False):
            fins[track] = _harness().run_parity(wl, normalize=normalize, prune=prune, track=track,
                                                check_state_every=4)
        differ = sum(1 for b in range(B) if fins[True][0][b].tobytes() != fins[False][0][b].tobytes())
        if not normalize:
            assert differ >= 2, (k, differ)


def test_gbs_simulation(torch_gpu):
    """Sec. 5: beam b(C+1), adjustment off - C = 3 single-token constraints, b = 5."""
    B, V, T, b, C = 6, 8000, 25, 5, 3
    cons = si.fixed_total_constraints(53, B, V, C, max_len=1)
    wl = si.Workload(B=B, k=b * (C + 1), V=V, T=T, seed=53, constraints=cons,
                     boost_tokens=[[w for p in s for w in p] for s in cons], boost_prob=0.05)
    _harness().run_parity(wl, adjust=False)


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("seed", range(8))
def test_16bit_logp_small(torch_gpu, seed, fmt):
    """16-bit log-probs (widened exactly, fp32 sums): odd V, so rows start at every 2-byte
    offset inside a 16-byte group; many exact ties, because 16-bit values collide."""
    rs = si.Stream(seed, 8)
    B = rs.randint(2, 5)
    k = [1, 3, 8, 13, 20, 33, 64, 5][seed % 8]
    V = max(k + 3, [67, 131, 1001, 1023, 2051, 4099, 515, 9001][(seed // 2 + seed) % 8])
    T = rs.randint(6, 12)
    wl = si.make_small(9500 + seed, B, k, V, T, max_phrases=5, max_len=4, dup_prob=0.35)
    wl.eos_switch = T // 2
    _harness().run_parity(wl, logp_format=fmt)


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_16bit_logp_config2_paper_setup(torch_gpu, fmt):
    wl = si.make_config(2, T=25)
    wl.eos_switch = 10
    _harness().run_parity(wl, logp_format=fmt, normalize=True, prune=20.0)


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_16bit_logp_config4(torch_gpu, fmt):
    """The headline shapes with 16-bit log-probs, 12 steps, all 64 sentences against the oracle."""
    wl = si.make_config(4, T=12)
    _harness().run_parity(wl, logp_format=fmt, check_state_every=4, progress=f"config4 {fmt}")


@pytest.mark.parametrize("k,V", [(64, 1 << 19), (2, 1 << 24)])
def test_widest_coordinates(torch_gpu, k, V):
    """The limits of the key packing, bits(k-1) + bits(V-1) + bits(64) = 32: the widest beam with
    the largest vocabulary it allows, and the largest vocabulary of all; 64 constraint tokens."""
    B, T = 1, 3
    cons = si.fixed_total_constraints(97, B, V, 64, max_len=4)
    wl = si.Workload(B=B, k=k, V=V, T=T, seed=97 + k, constraints=cons,
                     boost_tokens=[[w for p in s for w in p] for s in cons], boost_prob=0.3, boost_value=9.0)
    _harness().run_parity(wl, progress=f"k={k} V={V}")


@pytest.mark.parametrize("fmt", [None, "f16", "bf16"])
@pytest.mark.parametrize("B,k,V", [(2, 3, 9001), (1, 16, 20011), (1, 8, 33333), (3, 20, 12345)])
def test_small_batches_long_rows(torch_gpu, B, k, V, fmt):
    """Few rows of odd length and alignment, all three element types; hypotheses finish half
    way, so finished and empty rows take part too."""
    T = 10
    wl = si.make_small(9700 + k, B, k, V, T, max_phrases=5, max_len=3, dup_prob=0.3)
    wl.eos_switch = 4
    wl.eos_high = 1.0
    _harness().run_parity(wl, logp_format=fmt)


def test_two_contexts_on_their_own_streams(torch_gpu):
    """Two decodes at once, each context on a stream of its own (default priority), steps enqueued in
    turn without waiting: all work of a context goes to its stream and contexts share nothing."""
    from paper_1804_06609_amd.session import Session
    torch = torch_gpu
    wls = [si.make_small(9901, 3, 13, 2050, 10, max_phrases=4, max_len=3, dup_prob=0.3),
           si.make_small(9902, 2, 20, 4099, 10, max_phrases=5, max_len=2, dup_prob=0.2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    sess, beams = [], []
    for wl, st in zip(wls, streams):
        wl.eos_switch = 5
        toks, poff, soff = wl.csr()
        sess.append(Session(wl.B, wl.k, wl.V, wl.T, wl.eos_id, wl.pad_id, toks, poff, soff, stream=st))
        beams.append(oracle.BatchBeam(wl.k, wl.V, wl.constraints, wl.eos_id, wl.pad_id))
    torch.cuda.synchronize()
    for t in range(10):
        keep = []
        for wl, st, ses in zip(wls, streams, sess):
            with torch.cuda.stream(st):
                d = torch.from_numpy(wl.logp(t)).cuda()
                ses.step(d)
            keep.append(d)
        for wl, ses, bm in zip(wls, sess, beams):
            bm.step(wl.logp(t))
            tok, bp, sc, fl = ses.outputs()
            assert tok.tobytes() == bm.stacked("token").tobytes(), t
            assert bp.tobytes() == bm.stacked("backptr").tobytes(), t
            assert sc.tobytes() == bm.stacked("score").tobytes(), t
            assert fl.tobytes() == bm.stacked("flags").tobytes(), t
    for wl, ses, bm in zip(wls, sess, beams):
        got, want = ses.finalize(), bm.finalize(10)
        for g, w in zip(got, want):
            assert np.asarray(g).tobytes() == np.asarray(w).tobytes()
        ses.close()


def test_plain_c_caller(torch_gpu, tmp_path):
    """examples/decode_from_file.c (built with gcc, no binding in between) against the oracle."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "examples", "decode_from_file")
    assert os.path.exists(exe), "build it first: python -m paper_1804_06609_amd.build"
    wl = si.make_small(4711, 3, 4, 203, 9, max_phrases=3, max_len=3)
    wl.eos_switch = 4
    toks, poff, soff = wl.csr()
    lp = np.stack([wl.logp(t) for t in range(wl.T)])
    lp.tofile(tmp_path / "logp.bin")
    with open(tmp_path / "cons.txt", "w") as f:
        f.write(f"{len(toks)} {len(poff) - 1}\n" + " ".join(map(str, toks)) + "\n" +
                " ".join(map(str, poff)) + "\n" + " ".join(map(str, soff)) + "\n")
    out = subprocess.run([exe, str(wl.B), str(wl.k), str(wl.V), str(wl.T), str(wl.eos_id), str(wl.pad_id),
                          str(tmp_path / "logp.bin"), str(tmp_path / "cons.txt")],
                         capture_output=True, text=True, timeout=100)
    assert out.returncode == 0, out.stderr
    ob = oracle.BatchBeam(wl.k, wl.V, wl.constraints, wl.eos_id, wl.pad_id)
    want = []
    for t in range(wl.T):
        ob.step(lp[t])
        for b, bm in enumerate(ob.beams):
            cells = " ".join(f"{int(w)}/{int(h)}/{int(np.float32(s).view(np.uint32)):08x}"
                             for w, h, s in zip(bm.token, bm.backptr, bm.score))
            want.append(f"step {t} sent {b} : {cells}")
    ft, fl, fs, fst = ob.finalize(wl.T)
    for b in range(wl.B):
        tail = "".join(f" {int(w)}" for w in ft[b][:fl[b]])
        want.append(f"final {b} : {int(fst[b])} {int(fl[b])} {int(np.float32(fs[b]).view(np.uint32)):08x} :{tail}")
    assert out.stdout.strip().splitlines() == want


def test_call_order_errors(torch_gpu):
    """More than N steps, and an option change after the first step, are refused (no launch)."""
    import paper_1804_06609_amd as dba
    from paper_1804_06609_amd.session import Session
    wl = si.make_small(77, 2, 4, 64, 3)
    toks, poff, soff = wl.csr()
    ses = Session(wl.B, wl.k, wl.V, 3, wl.eos_id, wl.pad_id, toks, poff, soff)
    dev = torch_gpu.from_numpy(wl.logp(0)).cuda()
    with pytest.raises(dba.DbaError, match="unknown option"):
        dba.dba_set_option(ses.ctx, 9999, 1)
    with pytest.raises(dba.DbaError):
        dba.dba_set_option(ses.ctx, dba.DBA_OPT_MERGE_WAVES, 5)
    with pytest.raises(dba.DbaError, match="unknown log-prob format"):
        dba.dba_step_fmt(ses.ctx, dev.data_ptr(), 7)
    with pytest.raises(dba.DbaError, match="aligned"):
        dba.dba_step(ses.ctx, dev.data_ptr() + 2)
    assert dba.dba_steps_done(ses.ctx) == 0
    ses.step(dev)
    with pytest.raises(dba.DbaError, match="first step"):
        dba.dba_set_option(ses.ctx, dba.DBA_OPT_ADJUSTMENT, 0)
    mid = ses.finalize()                 # allowed after any number of steps
    assert mid[0].shape == (wl.B, 3)
    ses.step(dev)
    ses.step(dev)
    with pytest.raises(dba.DbaError):
        ses.step(dev)
    assert dba.dba_steps_done(ses.ctx) == 3
    ses.close()


def test_config1(torch_gpu):
    _harness().run_parity(si.make_config(1), progress="config1")


def test_config2(torch_gpu):
    _harness().run_parity(si.make_config(2), progress="config2")


def test_config3(torch_gpu):
    _harness().run_parity(si.make_config(3), progress="config3")


def test_config4(torch_gpu):
    """Headline shape, all 64 sentences, all 100 steps, the launch configuration bench.py times."""
    _harness().run_parity(si.make_config(4), check_state_every=5, progress="config4")


def test_config5(torch_gpu):
    """Full shape (B=128, k=64, V=50000), all 120 steps, EVERY sentence: the oracle's cost per sentence
    and step is ~0.3 s, so it followed all 128 sentences beforehand (tests/golden/make_config5_digests.py,
    oracle/ only) and left a chained digest of every step's tokens, parents, scores, flags and constraint
    state per sentence; the GPU outputs of all sentences go through the same chains here and must agree
    at every stored step and at the end of decoding.  Eight sentences are also followed by the oracle
    live, element by element, and must reproduce the stored digests themselves.
    DBA_TEST_CONFIG5_STEPS cuts the run short."""
    T = int(os.environ.get("DBA_TEST_CONFIG5_STEPS", "120"))
    wl = si.make_config(5, T=T)
    ntok = [wl.n_tokens(b) for b in range(wl.B)]
    sample = sorted({int(np.argmin(ntok)), int(np.argmax(ntok)), 0, 1, 63, 64, 126, 127})
    golden = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "config5_digests.txt")
    _harness().run_parity(wl, oracle_sentences=sample, check_state_every=5, progress="config5", golden=golden)


@pytest.mark.gpu
def test_reference_read_is_the_row_maximum():
    """The diagnostic read kernel (what the benchmark compares the step with) returns each row's
    largest element: a ragged last tile, several tiles per wave, -inf entries and a whole row of them."""
    import torch
    import paper_1804_06609_amd as dba
    rng = np.random.default_rng(77)
    for rows, V in ((3, 4), (5, 1000), (7, 32000), (4, 50000), (2, 1028)):
        x = rng.standard_normal((rows, V)).astype(np.float32)
        x[0, ::3] = -np.inf
        if rows > 2:
            x[2, :] = -np.inf
        d = torch.from_numpy(x).cuda()
        out = torch.full((rows,), 123.0, dtype=torch.float32, device="cuda")
        dba.dba_debug_row_max(d.data_ptr(), rows, V, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert out.cpu().numpy().tobytes() == x.max(axis=1).tobytes(), (rows, V)
    with pytest.raises(dba.DbaError):
        dba.dba_debug_row_max(d.data_ptr(), 2, 1027, out.data_ptr(), 0)
