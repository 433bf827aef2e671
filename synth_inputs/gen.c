/*
 * Seeded synthetic log-probability tensors for decoder-step stand-ins.
 *
 * This file only manufactures inputs: a counter-based random stream, a
 * Gaussian transform, and a row-wise log-softmax.  It contains nothing of the
 * beam-allocation method itself and is shared by every consumer of test data.
 *
 * Random stream: the 64-bit finaliser of SplitMix64 (Steele, Lea, Flood 2014)
 * applied to a counter built from (seed, step, row, pair).  Each pair of
 * vocabulary entries (2p, 2p+1) of a row takes one Box-Muller draw, so any
 * subset of rows can be produced alone and is bit-identical to the same rows
 * of a full tensor, whatever the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define GOLDEN 0x9E3779B97F4A7C15ull

static inline uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline double unit_open(uint64_t x)
{
    /* uniform in (0,1): 53 random bits, offset by half an ulp */
    return ((double)(x >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

uint64_t synth_mix64(uint64_t z) { return mix64(z); }

/*
 * out[(r - row0) * V + v] = float( log_softmax_v( N(0,1) + zbias[v] + extra ) )
 * for global rows r in [row0, row0 + nrows); row r belongs to sentence
 * r / rows_per_sent.  extra: for sentence b the entries
 * ex_off[b] .. ex_off[b+1]-1 add ex_val[i] to vocabulary entry ex_tok[i] in
 * every row of that sentence (ex_off may be NULL for none).
 * The softmax runs in double with a fixed left-to-right sum and is rounded to
 * float once.
 */
void synth_logp(uint64_t seed, uint64_t step, int64_t row0, int64_t nrows,
                int64_t rows_per_sent, int64_t V, const double *zbias,
                const int64_t *ex_off, const int32_t *ex_tok,
                const double *ex_val, float *out)
{
    const uint64_t step_key = mix64(seed + GOLDEN * (step + 1));
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)(V + 1) * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < nrows; ++i) {
            const int64_t r = row0 + i;
            const uint64_t row_key =
                mix64(step_key ^ ((uint64_t)(r + 1) * 0xD1B54A32D192ED03ull));
            for (int64_t p = 0; 2 * p < V; ++p) {
                const uint64_t c = row_key + GOLDEN * (uint64_t)(2 * p + 1);
                const double u1 = unit_open(mix64(c));
                const double u2 = unit_open(mix64(c + GOLDEN));
                const double rad = sqrt(-2.0 * log(u1));
                const double ang = two_pi * u2;
                z[2 * p] = rad * cos(ang);
                z[2 * p + 1] = rad * sin(ang); /* z has V+1 slots */
            }
            for (int64_t v = 0; v < V; ++v) z[v] += zbias[v];
            if (ex_off) {
                const int64_t b = r / rows_per_sent;
                for (int64_t e = ex_off[b]; e < ex_off[b + 1]; ++e)
                    z[ex_tok[e]] += ex_val[e];
            }
            double m = z[0];
            for (int64_t v = 1; v < V; ++v)
                if (z[v] > m) m = z[v];
            double acc = 0.0;
            for (int64_t v = 0; v < V; ++v) acc += exp(z[v] - m);
            const double lse = m + log(acc);
            float *o = out + (size_t)i * (size_t)V;
            for (int64_t v = 0; v < V; ++v) o[v] = (float)(z[v] - lse);
        }
        free(z);
    }
}
