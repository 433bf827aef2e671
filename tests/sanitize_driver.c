/*
 * Host-side sanitizer run over the CPU oracle and the input generator (test infrastructure).
 * Built by tests/test_sanitizers_cpu.py with -fsanitize=address,undefined and run once: seeded
 * small decodes through every variant of the oracle's step, the record of the best completed
 * hypothesis, both ends of decoding, the allocation on exhaustive small counts and the
 * constraint bookkeeping on random states.  Any out-of-bounds access, use of freed or
 * uninitialised stack memory the sanitizers can see, signed overflow or leak ends the run
 * with a non-zero status.  Prints a checksum so that the work cannot be optimised away.
 */
#include <stdio.h>

#include "../oracle/dba_oracle.c"
#include "../synth_inputs/gen.c"

static uint64_t rnd_state;
static uint64_t rnd(void)
{
    rnd_state += GOLDEN;
    return mix64(rnd_state);
}
static int rnd_int(int lo, int hi) { return lo + (int)(rnd() % (uint64_t)(hi - lo + 1)); }

int main(int argc, char **argv)
{
    const int n_seeds = argc > 1 ? atoi(argv[1]) : 300;
    uint64_t sum = 0;
    for (int seed = 0; seed < n_seeds; ++seed) {
        rnd_state = mix64(0xABCDEFull + (uint64_t)seed);
        const int k = rnd_int(1, 7), V = rnd_int(k + 4, 48), T = rnd_int(1, 9), N = T;
        const int eos = 2, pad = 0;
        int P = rnd_int(0, 4), C = 0;
        int32_t off[8] = {0}, tok[32];
        for (int j = 0; j < P; ++j) {
            const int len = rnd_int(1, 3);
            for (int i = 0; i < len; ++i) tok[C++] = rnd_int(4, V - 1);
            off[j + 1] = C;
        }
        const int adjust = rnd_int(0, 1), normalize = rnd_int(0, 1);
        const float prune = rnd_int(0, 2) == 0 ? -1.0f : (float)rnd_int(0, 6);
        /* beam */
        float *score = malloc(sizeof(float) * k), *o_sc = malloc(sizeof(float) * k);
        uint64_t *met = calloc(k, 8), *o_met = malloc(8 * k);
        int32_t *ip = malloc(4 * k), *iq = calloc(k, 4), *len = calloc(k, 4);
        int32_t *o_tok = malloc(4 * k), *o_bp = malloc(4 * k), *o_ip = malloc(4 * k), *o_iq = malloc(4 * k),
                *o_len = malloc(4 * k);
        uint8_t *fin = calloc(k, 1), *o_fl = malloc(k);
        int32_t *hist_tok = malloc(4 * (size_t)T * k), *hist_bp = malloc(4 * (size_t)T * k);
        for (int h = 0; h < k; ++h) {
            score[h] = h == 0 ? 0.0f : -INFINITY;
            ip[h] = -1;
        }
        uint8_t *flags = malloc(k);
        int32_t rec_int[4] = {0, 0, 0, 0};
        float rec_flt[2] = {0.0f, 0.0f};
        double *zb = malloc(sizeof(double) * V);
        float *logp = malloc(sizeof(float) * (size_t)k * V);
        for (int v = 0; v < V; ++v) zb[v] = -1.1 * log((double)(1 + (v * 7 + seed) % V));
        const int cap = k * (P + 2) > 0 ? k * (P + 2) : 1;
        int64_t *d_flat = malloc(8 * (size_t)cap);
        int32_t *d_bank = malloc(4 * (size_t)cap), d_cnt[65], d_alloc[65], d_n = 0, done = 0;
        for (int t = 0; t < T; ++t) {
            zb[eos] = t >= T / 2 ? 1.0 : -30.0;
            const int64_t ex_off[2] = {0, C > 0 ? 1 : 0};
            const int32_t ex_tok[1] = {C > 0 ? tok[0] : 0};
            const double ex_val[1] = {4.0};
            synth_logp(77 + (uint64_t)seed, (uint64_t)t, 0, k, k, V, zb, ex_off, ex_tok, ex_val, logp);
            if (dba_oracle_step(k, V, eos, pad, P, off, tok, score, met, ip, iq, fin, len, logp, o_tok, o_bp,
                                o_sc, o_fl, o_met, o_ip, o_iq, o_len, &d_n, d_flat, d_bank, d_cnt, d_alloc, adjust,
                                normalize, prune, &done) != 0)
                return 2;
            dba_oracle_track_completed(k, t, o_sc, o_fl, o_len, normalize, rec_int, rec_flt);
            for (int h = 0; h < k; ++h) {
                score[h] = o_sc[h];
                met[h] = o_met[h];
                ip[h] = o_ip[h];
                iq[h] = o_iq[h];
                len[h] = o_len[h];
                fin[h] = (uint8_t)(o_fl[h] & FLAG_FINISHED);
                flags[h] = o_fl[h];
                hist_tok[(size_t)t * k + h] = o_tok[h];
                hist_bp[(size_t)t * k + h] = o_bp[h];
                sum += (uint64_t)o_tok[h] * 31u + (uint64_t)(o_bp[h] + 1);
            }
            sum += (uint64_t)d_n + (uint64_t)done;
        }
        int32_t *nmet = malloc(4 * k), *out_tokens = malloc(4 * (size_t)N), out_len, out_status;
        float out_score;
        for (int h = 0; h < k; ++h) nmet[h] = __builtin_popcountll(met[h]);
        dba_oracle_finalize(k, T, N, pad, hist_tok, hist_bp, score, flags, len, nmet, out_tokens, &out_len, &out_score,
                            &out_status, normalize);
        sum += (uint64_t)out_len + (uint64_t)out_status;
        dba_oracle_finalize_tracked(k, T, N, pad, hist_tok, hist_bp, score, flags, len, nmet, out_tokens, &out_len,
                                    &out_score, &out_status, normalize, rec_int, rec_flt);
        sum += (uint64_t)out_len + (uint64_t)out_status;
        /* constraint bookkeeping on random (valid) states */
        if (P > 0) {
            for (int r = 0; r < 20; ++r) {
                uint64_t m = 0, m2;
                int ipj = -1, iqj = 0, a, b, nn;
                int32_t nxt[64];
                for (int j = 0; j < P; ++j) {
                    const int l = off[j + 1] - off[j];
                    const int q = rnd_int(0, 2) == 0 ? l : 0;
                    for (int i = 0; i < q; ++i) m |= (uint64_t)1 << (off[j] + i);
                }
                const int j = rnd_int(0, P - 1);
                if (off[j + 1] - off[j] > 1 && !((m >> off[j]) & 1)) {
                    ipj = j;
                    iqj = rnd_int(1, off[j + 1] - off[j] - 1);
                    for (int i = 0; i < iqj; ++i) m |= (uint64_t)1 << (off[j] + i);
                }
                dba_oracle_add(P, off, tok, m, ipj, iqj, rnd_int(-1, V - 1), &m2, &a, &b, nxt, &nn);
                sum += m2 + (uint64_t)(a + 1) + (uint64_t)b + (uint64_t)nn;
            }
        }
        free(score); free(o_sc); free(met); free(o_met); free(ip); free(iq); free(len); free(o_tok); free(o_bp);
        free(o_ip); free(o_iq); free(o_len); free(fin); free(o_fl); free(hist_tok); free(hist_bp); free(flags);
        free(zb); free(logp); free(d_flat); free(d_bank); free(nmet); free(out_tokens);
    }
    /* allocation: exhaustive small counts, both forms; then 64 constraint tokens */
    for (int k = 1; k <= 6; ++k)
        for (int C = 0; C <= 3; ++C) {
            int32_t cnt[4], alloc[4];
            const int lim = k + 2;
            int total = 1;
            for (int i = 0; i <= C; ++i) total *= lim;
            for (int code = 0; code < total; ++code) {
                int x = code;
                for (int i = 0; i <= C; ++i) {
                    cnt[i] = x % lim;
                    x /= lim;
                }
                dba_oracle_allocate(k, C, cnt, alloc);
                for (int i = 0; i <= C; ++i) sum += (uint64_t)alloc[i];
                dba_oracle_allocate_fixed(k, C, cnt, alloc);
                for (int i = 0; i <= C; ++i) sum += (uint64_t)alloc[i];
            }
        }
    {
        int32_t cnt[65], alloc[65];
        for (int r = 0; r < 200; ++r) {
            for (int i = 0; i < 65; ++i) cnt[i] = rnd_int(0, 3) == 0 ? rnd_int(0, 70) : 0;
            dba_oracle_allocate(rnd_int(1, 64), 64, cnt, alloc);
            for (int i = 0; i < 65; ++i) sum += (uint64_t)alloc[i];
        }
    }
    printf("sanitize_driver ok %llu\n", (unsigned long long)sum);
    return 0;
}
