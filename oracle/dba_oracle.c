/*
 * CPU oracle for one time step of k-best extraction with Dynamic Beam
 * Allocation (Post & Vilar 2018, Alg. 2 and Sections 3.1-3.3), for ONE
 * sentence.  Sentences never interact, so a batch is a loop over this.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain statement of what the
 * step computes; the GPU library shares no code with it and never calls it.
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may use it.
 *
 * DBA is a heuristic selection procedure, not a shortcut to a closed form, so
 * the oracle is the algorithm itself, in the paper's order:
 *   scores (Sec. 2: entry (i,j) extends hypothesis i by word j)
 *   -> candidates from three sources (Sec. 3.1 items 1-3)
 *   -> constraint bookkeeping incl. unwinding (Sec. 3.1, last paragraph)
 *   -> banks by number of met constraints (Sec. 3.1) and allocation with
 *      adjustment (Sec. 3.2)
 *   -> new beam, best first (Sec. 3.1, first paragraph)
 *   -> no end-of-sentence before all constraints are met (Sec. 3.3).
 * Where the paper leaves a point open the reading taken is written at the
 * place it applies.
 *
 * Precision: a score is ONE fp32 addition prev + logp (round to nearest even);
 * all comparisons are on those sums; equal sums are ordered by the lower flat
 * coordinate h*V + w.
 *
 * Pins: parity of the full step against the paper is unpinned (the paper
 * prints no numeric worked example).  What is pinned by tests: C=0 reduces
 * to textbook top-k; the figure captions' allocation facts (k=5, C=4);
 * sum(alloc) = min(k, #candidates); alloc <= count; independent brute-force
 * enumeration on tiny sizes; trajectory invariants (met count monotone except
 * on unwinding, finished implies all met).  Unpinned readings: the C+1
 * divisor of the base bank size, donor order and neighbour preference of the
 * adjustment, first-tokens of other phrases being expandable while one phrase
 * is in progress, the lowest-phrase-index rule and restart-after-unwind of
 * add().
 *
 * Variants of the experimental set-up (Sec. 4, Sec. 5, Sec. 6.3), each off by
 * default and switched by an argument of dba_oracle_step: allocation without
 * adjustment (the GBS simulation of Sec. 5), scores of completed hypotheses
 * divided by their length while they sit on the beam (Sec. 4; Fig. 9 caption),
 * threshold pruning against the best completed hypothesis (Sec. 4, Sec. 6.3)
 * and the all-completed stopping test (Sec. 4).  Pinned by tests: the
 * stored score of a completed hypothesis equals the fp32 sum of the log-probs
 * along its back-pointer path divided by its length; a pruned step equals the
 * unpruned step with the losers struck out; survivors lie within the
 * threshold of the best completed one; brute-force enumeration.  Unpinned
 * readings: raw sums decide the selection inside the step in which a
 * hypothesis completes; the pruning cut-off is the fp32 difference best -
 * threshold and a score equal to it survives.
 *
 * Completed hypotheses that leave the beam (Sec. 3.3: what decoding returns is
 * the best-scoring hypothesis among the finished ones).  A completed hypothesis sits in the topmost
 * bank and can lose its slot there to candidates with higher sums.  Reading
 * of the bare algorithm (dba_oracle_finalize): only the final beam is
 * searched, so such a hypothesis is forgotten.  Variant
 * (dba_oracle_track_completed + dba_oracle_finalize_tracked): a record of the
 * best completed hypothesis seen on any beam is kept from step to step and
 * returned at the end.  Pinned by tests: the returned hypothesis scores at
 * least as well as every completed hypothesis that ever sat on a beam, found
 * by walking the recorded beams, and its tokens are the back-trace from the
 * step and slot where it was seen; with no drop-out both readings agree.
 * Unpinned: among equal scores the earliest step, then the lowest slot wins.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define DBA_ORACLE_MAX_TOKENS 64

#define FLAG_FINISHED 1
#define FLAG_DEAD 2

/* ---- constraint state of one hypothesis (Sec. 3.1; Fig. 2 caption) -------
 * met[i] says whether constraint token i (in phrase order) is marked met.
 * A phrase is generated in order, so its met tokens are a prefix of it; at
 * most one phrase is under way: phrase `ip` has its first `iq` tokens met
 * (ip = -1: none under way). */
typedef struct {
    unsigned char met[DBA_ORACLE_MAX_TOKENS];
    int ip, iq;
} cstate;

typedef struct {
    int P, C;
    const int32_t *off; /* [P+1] token offsets of the phrases */
    const int32_t *tok; /* [C] */
} cons_t;

static int count_met(const cons_t *c, const cstate *s)
{
    int n = 0;
    for (int i = 0; i < c->C; ++i) n += s->met[i] ? 1 : 0;
    return n;
}

static int phrase_complete(const cons_t *c, const cstate *s, int j)
{
    for (int i = c->off[j]; i < c->off[j + 1]; ++i)
        if (!s->met[i]) return 0;
    return 1;
}

/*
 * constraints.add(w) of Alg. 2: the state after the hypothesis emits w.
 * Reading: (1) the phrase under way advances if w is its next token;
 * (2) otherwise a phrase under way is unwound - every token of it goes back
 * to unmet (Sec. 3.1: a token that does not continue a begun phrase resets
 * the tokens of that phrase marked met) - and then (3) w may start a phrase:
 * among phrases that are not complete, the one with the lowest index whose
 * first token is w.  One emitted token advances at most one phrase.
 */
static void cstate_add(const cons_t *c, cstate *s, int w)
{
    if (s->ip >= 0) {
        const int pos = c->off[s->ip] + s->iq;
        if (c->tok[pos] == w) {
            s->met[pos] = 1;
            s->iq += 1;
            if (c->off[s->ip] + s->iq == c->off[s->ip + 1]) {
                s->ip = -1;
                s->iq = 0;
            }
            return;
        }
        for (int i = c->off[s->ip]; i < c->off[s->ip + 1]; ++i) s->met[i] = 0;
        s->ip = -1;
        s->iq = 0;
    }
    for (int j = 0; j < c->P; ++j) {
        if (phrase_complete(c, s, j)) continue;
        if (c->tok[c->off[j]] != w) continue;
        s->met[c->off[j]] = 1;
        if (c->off[j + 1] - c->off[j] > 1) {
            s->ip = j;
            s->iq = 1;
        }
        return;
    }
}

/*
 * "All unmet constraints" of a hypothesis (Alg. 2 inner loop; Sec. 3.1 item 2)
 * under in-order phrases: the next token of the phrase under way, and the
 * first token of every phrase that is neither complete nor under way.
 * Interior tokens of a phrase not yet begun cannot be placed.
 * Returns the number of tokens written to out (at most P).
 */
static int cstate_next_tokens(const cons_t *c, const cstate *s, int32_t *out)
{
    int n = 0;
    for (int j = 0; j < c->P; ++j) {
        if (j == s->ip)
            out[n++] = c->tok[c->off[j] + s->iq];
        else if (!phrase_complete(c, s, j))
            out[n++] = c->tok[c->off[j]];
    }
    return n;
}

/* ---- allocation (Sec. 3.2) ------------------------------------------------
 * k slots over banks 0..C.  The printed base size floor(k/C) cannot be meant
 * literally for C+1 banks (it over-fills the beam and divides by zero at
 * C=0); reading: every bank gets floor(k/(C+1)) and the remainder goes to the
 * topmost bank C - which gives the one-slot-per-bank split of the k=5, C=4
 * figures and a single bank of k for C=0.
 * Adjustment (given only as a sketch): each bank holding more slots than
 * candidates, taken in ascending order, keeps what it can fill and hands the
 * rest to banks with more candidates than slots, nearest first, the higher
 * neighbour before the lower at equal distance, as much as each can take.
 * Slots nobody can take are dropped, so the beam is filled up to
 * min(k, #candidates). */
void dba_oracle_allocate(int k, int C, const int32_t *cnt, int32_t *alloc)
{
    const int base = k / (C + 1);
    for (int b = 0; b <= C; ++b) alloc[b] = base;
    alloc[C] += k - base * (C + 1);
    for (int b = 0; b <= C; ++b) {
        int extra = alloc[b] - cnt[b];
        if (extra <= 0) continue;
        alloc[b] = cnt[b];
        for (int d = 1; d <= C && extra > 0; ++d) {
            const int nb[2] = {b + d, b - d};
            for (int s = 0; s < 2 && extra > 0; ++s) {
                const int x = nb[s];
                if (x < 0 || x > C) continue;
                if (cnt[x] > alloc[x]) {
                    int g = cnt[x] - alloc[x];
                    if (g > extra) g = extra;
                    alloc[x] += g;
                    extra -= g;
                }
            }
        }
    }
}

/* Allocation with the adjustment switched off (Sec. 5, the simulated GBS
 * baseline: the room of a bank does not change): the base split of Sec. 3.2;
 * a bank with fewer candidates than slots leaves the rest of its slots empty. */
void dba_oracle_allocate_fixed(int k, int C, const int32_t *cnt, int32_t *alloc)
{
    const int base = k / (C + 1);
    for (int b = 0; b <= C; ++b) alloc[b] = base;
    alloc[C] += k - base * (C + 1);
    for (int b = 0; b <= C; ++b)
        if (alloc[b] > cnt[b]) alloc[b] = cnt[b];
}

/* state transition alone, for direct tests of add() and the expandable set */
void dba_oracle_add(int P, const int32_t *off, const int32_t *tok, uint64_t met_in,
                    int ip_in, int iq_in, int w, uint64_t *met_out, int *ip_out, int *iq_out,
                    int32_t *next_out, int *n_next_out)
{
    cons_t c = {P, off[P], off, tok};
    cstate s;
    memset(&s, 0, sizeof s);
    for (int i = 0; i < c.C; ++i) s.met[i] = (unsigned char)((met_in >> i) & 1u);
    s.ip = ip_in;
    s.iq = iq_in;
    if (next_out) *n_next_out = cstate_next_tokens(&c, &s, next_out);
    if (w >= 0) cstate_add(&c, &s, w);
    uint64_t m = 0;
    for (int i = 0; i < c.C; ++i)
        if (s.met[i]) m |= (uint64_t)1 << i;
    *met_out = m;
    *ip_out = s.ip;
    *iq_out = s.iq;
}

typedef struct {
    int h, w;
    long long flat;
    float s;
    cstate st;
    int bank;
    int chosen;
} cand_t;

/* (score descending, flat coordinate ascending): is a before b? */
static int cand_before(const cand_t *a, const cand_t *b)
{
    if (a->s > b->s) return 1;
    if (a->s < b->s) return 0;
    return a->flat < b->flat;
}

static void sort_cands(cand_t **v, int n)
{
    for (int i = 1; i < n; ++i) {
        cand_t *x = v[i];
        int j = i - 1;
        while (j >= 0 && cand_before(x, v[j])) {
            v[j + 1] = v[j];
            --j;
        }
        v[j + 1] = x;
    }
}

/*
 * One DBA step of one sentence.
 *
 * in : k hypotheses (slot order = row order of logp): cumulative score
 *      (-inf = empty slot), met mask (bit i = constraint token i), phrase
 *      under way (ip, iq), finished flag, length; logp[k][V].
 * out: the new beam, best first (token, parent slot, score, flags, state,
 *      length); unused slots: token pad, parent -1, score -inf, flag DEAD.
 * dbg_* (each may be NULL): candidate count, per-candidate flat/bank (room for
 *      k*(P+2)), bank counts and final allocation [C+1].
 * Variants (the paper's defaults for its experiments differ from the bare
 * algorithm; 1, 0, negative, NULL give the bare algorithm):
 *   adjust              0: no adjustment of the bank sizes (Sec. 5).
 *   normalize_finished  1: a hypothesis that generates end-of-sentence in this
 *      step is stored with score = sum / length (one fp32 division, the length
 *      counts end-of-sentence) and keeps that score while it stays on the beam
 *      (Sec. 4; Fig. 9 caption: only finished hypotheses are normalised).
 *      Reading: inside this step it still competes with its raw sum - the
 *      entry of the scores matrix - and the new beam is ordered by those sums.
 *   prune_threshold     >= 0: after the new beam is formed, every hypothesis,
 *      completed or not, whose stored score is below (best stored score of a
 *      completed hypothesis on the new beam) - threshold is removed (Sec. 4);
 *      the rest close ranks in order.  No completed hypothesis: no pruning.
 *   out_all_finished    receives the stopping tests as two bits: 1 when the new
 *      beam is not empty and all its hypotheses are completed (Sec. 4), 2 when
 *      at least one hypothesis on it is completed (the early stopping that
 *      Sec. 6.3 mentions as the alternative to pruning).
 * Returns 0, or -1 on bad arguments.
 */
int dba_oracle_step(int k, int V, int eos_id, int pad_id, int P, const int32_t *phrase_off,
                    const int32_t *tokens, const float *prev_score, const uint64_t *met_in,
                    const int32_t *ip_in, const int32_t *iq_in, const uint8_t *fin_in,
                    const int32_t *len_in, const float *logp, int32_t *out_token,
                    int32_t *out_backptr, float *out_score, uint8_t *out_flags,
                    uint64_t *out_met, int32_t *out_ip, int32_t *out_iq, int32_t *out_len,
                    int32_t *dbg_ncand, int64_t *dbg_flat, int32_t *dbg_bank, int32_t *dbg_cnt,
                    int32_t *dbg_alloc, int adjust, int normalize_finished, float prune_threshold,
                    int32_t *out_all_finished)
{
    if (k < 1 || V < 1 || P < 0) return -1;
    cons_t c = {P, phrase_off[P], phrase_off, tokens};
    if (c.C > DBA_ORACLE_MAX_TOKENS) return -1;
    const int C = c.C;
    const float NEG_INF = -INFINITY;

    cstate *st = (cstate *)calloc((size_t)k, sizeof(cstate));
    int *nmet = (int *)calloc((size_t)k, sizeof(int));
    for (int h = 0; h < k; ++h) {
        for (int i = 0; i < C; ++i) st[h].met[i] = (unsigned char)((met_in[h] >> i) & 1u);
        st[h].ip = ip_in[h];
        st[h].iq = iq_in[h];
        nmet[h] = count_met(&c, &st[h]);
    }

    /* scores: s[h][w] = prev[h] + logp[h][w], one fp32 add (Sec. 2).
     * An empty slot has no extensions.  A finished hypothesis stays on the
     * beam unchanged (Sec. 4: decoding runs until all hypotheses on the beam
     * are completed): its only extension is the pad token at log-prob 0.
     * End-of-sentence is impossible before all constraints are met (Sec. 3.3). */
    float *s = (float *)malloc((size_t)k * (size_t)V * sizeof(float));
    for (int h = 0; h < k; ++h) {
        float *row = s + (size_t)h * V;
        const float *lp = logp + (size_t)h * V;
        if (prev_score[h] == NEG_INF) {
            for (int w = 0; w < V; ++w) row[w] = NEG_INF;
        } else if (fin_in[h]) {
            for (int w = 0; w < V; ++w) row[w] = NEG_INF;
            row[pad_id] = prev_score[h] + 0.0f;
        } else {
            for (int w = 0; w < V; ++w) row[w] = prev_score[h] + lp[w];
            if (nmet[h] < C) row[eos_id] = NEG_INF;
        }
    }

    const int cap = k * (P + 2);
    cand_t *cand = (cand_t *)calloc((size_t)cap, sizeof(cand_t));
    int n = 0;

#define ADD_CAND(hh, ww)                                                     \
    do {                                                                     \
        const long long fl_ = (long long)(hh) * V + (ww);                    \
        int dup_ = 0;                                                        \
        for (int q_ = 0; q_ < n; ++q_)                                       \
            if (cand[q_].flat == fl_) dup_ = 1;                              \
        if (!dup_ && s[fl_] > NEG_INF) {                                     \
            cand[n].h = (hh);                                                \
            cand[n].w = (ww);                                                \
            cand[n].flat = fl_;                                              \
            cand[n].s = s[fl_];                                              \
            ++n;                                                             \
        }                                                                    \
    } while (0)

    /* source 1: the k best entries of the whole matrix (Sec. 3.1 item 1):
     * k times the best entry not yet taken; strict '>' on an ascending scan
     * keeps the lowest coordinate among equals. */
    {
        unsigned char *taken = (unsigned char *)calloc((size_t)k * V, 1);
        for (int r = 0; r < k; ++r) {
            long long best = -1;
            for (long long f = 0; f < (long long)k * V; ++f) {
                if (taken[f]) continue;
                if (best < 0 || s[f] > s[best]) best = f;
            }
            if (best < 0 || !(s[best] > NEG_INF)) break;
            taken[best] = 1;
            ADD_CAND((int)(best / V), (int)(best % V));
        }
        free(taken);
    }
    /* sources 2 and 3, hypothesis by hypothesis (Alg. 2 loop over the beam) */
    for (int h = 0; h < k; ++h) {
        if (prev_score[h] == NEG_INF) continue;
        if (!fin_in[h]) {
            int32_t nxt[DBA_ORACLE_MAX_TOKENS];
            const int nn = cstate_next_tokens(&c, &st[h], nxt);
            for (int i = 0; i < nn; ++i) ADD_CAND(h, nxt[i]); /* item 2 */
        }
        int best = 0;
        const float *row = s + (size_t)h * V;
        for (int w = 1; w < V; ++w)
            if (row[w] > row[best]) best = w;
        ADD_CAND(h, best); /* item 3 */
    }
#undef ADD_CAND

    /* bookkeeping of every candidate and its bank (Sec. 3.1) */
    int32_t cnt[DBA_ORACLE_MAX_TOKENS + 1], alloc[DBA_ORACLE_MAX_TOKENS + 1];
    for (int b = 0; b <= C; ++b) cnt[b] = 0;
    for (int i = 0; i < n; ++i) {
        cand[i].st = st[cand[i].h];
        if (!fin_in[cand[i].h]) cstate_add(&c, &cand[i].st, cand[i].w);
        cand[i].bank = count_met(&c, &cand[i].st);
        cnt[cand[i].bank] += 1;
    }
    if (adjust)
        dba_oracle_allocate(k, C, cnt, alloc);
    else
        dba_oracle_allocate_fixed(k, C, cnt, alloc);

    /* per bank: best first, take as many as the bank was given */
    cand_t **order = (cand_t **)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(cand_t *));
    cand_t **sel = (cand_t **)malloc((size_t)k * sizeof(cand_t *));
    int nsel = 0;
    for (int b = 0; b <= C; ++b) {
        int m = 0;
        for (int i = 0; i < n; ++i)
            if (cand[i].bank == b) order[m++] = &cand[i];
        sort_cands(order, m);
        for (int i = 0; i < m && i < alloc[b]; ++i) {
            order[i]->chosen = 1;
            if (nsel < k) sel[nsel++] = order[i];
        }
    }
    /* the beam is kept best first (Sec. 3.1) */
    sort_cands(sel, nsel);

    for (int i = 0; i < k; ++i) {
        if (i < nsel) {
            const cand_t *x = sel[i];
            const int pf = fin_in[x->h] ? 1 : 0;
            const int f = pf || x->w == eos_id;
            out_token[i] = x->w;
            out_backptr[i] = x->h;
            out_score[i] = x->s;
            out_flags[i] = (uint8_t)(f ? FLAG_FINISHED : 0);
            uint64_t m = 0;
            for (int q = 0; q < C; ++q)
                if (x->st.met[q]) m |= (uint64_t)1 << q;
            out_met[i] = m;
            out_ip[i] = x->st.ip;
            out_iq[i] = x->st.iq;
            out_len[i] = pf ? len_in[x->h] : len_in[x->h] + 1;
            if (normalize_finished && f && !pf) out_score[i] = out_score[i] / (float)out_len[i];
        } else {
            out_token[i] = pad_id;
            out_backptr[i] = -1;
            out_score[i] = NEG_INF;
            out_flags[i] = FLAG_DEAD;
            out_met[i] = 0;
            out_ip[i] = -1;
            out_iq[i] = 0;
            out_len[i] = 0;
        }
    }

    /* threshold pruning (Sec. 4, Sec. 6.3) */
    if (prune_threshold >= 0.0f) {
        int have = 0;
        float best = NEG_INF;
        for (int i = 0; i < nsel; ++i)
            if ((out_flags[i] & FLAG_FINISHED) && (!have || out_score[i] > best)) {
                best = out_score[i];
                have = 1;
            }
        if (have) {
            const float cut = best - prune_threshold;
            int m = 0;
            for (int i = 0; i < nsel; ++i) {
                if (!(out_score[i] >= cut)) continue;
                out_token[m] = out_token[i];
                out_backptr[m] = out_backptr[i];
                out_score[m] = out_score[i];
                out_flags[m] = out_flags[i];
                out_met[m] = out_met[i];
                out_ip[m] = out_ip[i];
                out_iq[m] = out_iq[i];
                out_len[m] = out_len[i];
                ++m;
            }
            for (int i = m; i < nsel; ++i) {
                out_token[i] = pad_id;
                out_backptr[i] = -1;
                out_score[i] = NEG_INF;
                out_flags[i] = FLAG_DEAD;
                out_met[i] = 0;
                out_ip[i] = -1;
                out_iq[i] = 0;
                out_len[i] = 0;
            }
            nsel = m;
        }
    }
    /* stopping tests (Sec. 4; Sec. 6.3) */
    if (out_all_finished) {
        int all = nsel > 0, any = 0;
        for (int i = 0; i < nsel; ++i) {
            if (!(out_flags[i] & FLAG_FINISHED)) all = 0;
            else any = 1;
        }
        *out_all_finished = all | (any << 1);
    }

    if (dbg_ncand) *dbg_ncand = n;
    for (int i = 0; i < n; ++i) {
        if (dbg_flat) dbg_flat[i] = cand[i].flat;
        if (dbg_bank) dbg_bank[i] = cand[i].bank;
    }
    for (int b = 0; b <= C; ++b) {
        if (dbg_cnt) dbg_cnt[b] = cnt[b];
        if (dbg_alloc) dbg_alloc[b] = alloc[b];
    }

    free(sel);
    free(order);
    free(cand);
    free(s);
    free(nmet);
    free(st);
    return 0;
}

/*
 * End of decoding for one sentence (Sec. 3.3: the answer is the best-scoring
 * finished hypothesis; Sec. 4: completed hypotheses are ranked by the
 * cumulative score divided by the number of words).
 * Reading: a hypothesis is completed when it has generated end-of-sentence
 * (which implies all constraints met); the length counts that token; the
 * quotient is one fp32 division; equal quotients go to the lower slot.  With
 * no completed hypothesis the status is 0 and the fallback is the live slot
 * with most constraints met, then best raw score, then lowest slot.
 *
 * scores_normalized = 1: the beam already holds sum/length for completed
 * hypotheses (normalize_finished of the step), so they are ranked by the
 * stored score as it is.
 *
 * hist_token / hist_backptr: [T][k] records of the T steps taken.
 * final beam: score, flags, len, nmet [k].
 * out_tokens [N] (pad-filled), out_len, out_score (as stored on the beam), out_status.
 */
int dba_oracle_finalize(int k, int T, int N, int pad_id, const int32_t *hist_token,
                        const int32_t *hist_backptr, const float *score, const uint8_t *flags,
                        const int32_t *len, const int32_t *nmet, int32_t *out_tokens,
                        int32_t *out_len, float *out_score, int32_t *out_status,
                        int scores_normalized)
{
    for (int i = 0; i < N; ++i) out_tokens[i] = pad_id;
    *out_len = 0;
    *out_score = -INFINITY;
    *out_status = 0;
    if (T < 1) return 0;
    int best = -1;
    float bestq = 0.0f;
    for (int h = 0; h < k; ++h) {
        if ((flags[h] & FLAG_DEAD) || !(flags[h] & FLAG_FINISHED)) continue;
        const float q = scores_normalized ? score[h] : score[h] / (float)len[h];
        if (best < 0 || q > bestq) {
            best = h;
            bestq = q;
        }
    }
    if (best >= 0) {
        *out_status = 1;
    } else {
        for (int h = 0; h < k; ++h) {
            if (flags[h] & FLAG_DEAD) continue;
            if (best < 0 || nmet[h] > nmet[best] ||
                (nmet[h] == nmet[best] && score[h] > score[best]))
                best = h;
        }
        if (best < 0) return 0;
    }
    *out_len = len[best];
    *out_score = score[best];
    int slot = best;
    for (int t = T - 1; t >= 0; --t) {
        if (t < len[best] && t < N) out_tokens[t] = hist_token[(size_t)t * k + slot];
        slot = hist_backptr[(size_t)t * k + slot];
    }
    return 0;
}


/*
 * Record of the best completed hypothesis seen so far (variant; see the header).
 * Called after every step with the new beam (after pruning, if any) of step t
 * (0-based).  A completed hypothesis is ranked by its score per word (Sec. 4):
 * the stored score itself when the beam already holds sum/length
 * (scores_normalized), else one fp32 division of the stored sum by the length.
 * The record changes only for a strictly better value, so a hypothesis that
 * is carried along on the beam is recorded where it first appeared, and among
 * equal values the earliest step and then the lowest slot win.
 * rec_int = {have, step, slot, length}, rec_flt = {value per word, stored score}.
 */
void dba_oracle_track_completed(int k, int t, const float *score, const uint8_t *flags,
                                const int32_t *len, int scores_normalized, int32_t *rec_int,
                                float *rec_flt)
{
    for (int h = 0; h < k; ++h) {
        if ((flags[h] & FLAG_DEAD) || !(flags[h] & FLAG_FINISHED)) continue;
        const float q = scores_normalized ? score[h] : score[h] / (float)len[h];
        if (!rec_int[0] || q > rec_flt[0]) {
            rec_int[0] = 1;
            rec_int[1] = t;
            rec_int[2] = h;
            rec_int[3] = len[h];
            rec_flt[0] = q;
            rec_flt[1] = score[h];
        }
    }
}

/*
 * End of decoding with the record above: the recorded hypothesis is returned
 * (status 1; length and score as stored when it was seen; tokens by following
 * the back-pointers from its step and slot).  Without a record nothing was
 * ever completed and the fallback of dba_oracle_finalize applies.
 */
int dba_oracle_finalize_tracked(int k, int T, int N, int pad_id, const int32_t *hist_token,
                                const int32_t *hist_backptr, const float *score,
                                const uint8_t *flags, const int32_t *len, const int32_t *nmet,
                                int32_t *out_tokens, int32_t *out_len, float *out_score,
                                int32_t *out_status, int scores_normalized, const int32_t *rec_int,
                                const float *rec_flt)
{
    if (!rec_int[0] || T < 1)
        return dba_oracle_finalize(k, T, N, pad_id, hist_token, hist_backptr, score, flags, len, nmet,
                                   out_tokens, out_len, out_score, out_status, scores_normalized);
    for (int i = 0; i < N; ++i) out_tokens[i] = pad_id;
    *out_status = 1;
    *out_len = rec_int[3];
    *out_score = rec_flt[1];
    int slot = rec_int[2];
    for (int t = rec_int[1]; t >= 0; --t) {
        if (t < rec_int[3] && t < N) out_tokens[t] = hist_token[(size_t)t * k + slot];
        slot = hist_backptr[(size_t)t * k + slot];
    }
    return 0;
}
