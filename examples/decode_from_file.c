/*
 * libdba from plain C: runs dba_init / dba_step / dba_finalize on log-probs read from a file
 * and prints every step's beam, so that the C ABI can be exercised (and checked) without any
 * binding.  Alg. 1 of Post & Vilar (2018) with kbest = Alg. 2; the "decoder" is the file.
 *
 *   decode_from_file B k V N eos_id pad_id logp.bin constraints.txt
 *
 * logp.bin         N x [B,k,V] fp32, step after step
 * constraints.txt  whitespace-separated integers: n_tokens n_phrases, then the tokens, then
 *                  the n_phrases+1 phrase offsets, then the B+1 sentence offsets
 *
 * Output, one line per step and sentence: "step t sent b : token/parent/scorebits ..." and at
 * the end "final b : status len scorebits : tokens".
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/dba.h"

#define HIP_OK(x)                                                                      \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                                  \
        }                                                                              \
    } while (0)

static int32_t *read_ints(FILE *f, int n)
{
    int32_t *v = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    for (int i = 0; i < n; ++i)
        if (fscanf(f, "%d", &v[i]) != 1) {
            free(v);
            return NULL;
        }
    return v;
}

int main(int argc, char **argv)
{
    if (argc != 9) {
        fprintf(stderr, "usage: %s B k V N eos_id pad_id logp.bin constraints.txt\n", argv[0]);
        return 1;
    }
    const int B = atoi(argv[1]), k = atoi(argv[2]), V = atoi(argv[3]), N = atoi(argv[4]);
    const int eos_id = atoi(argv[5]), pad_id = atoi(argv[6]);

    FILE *fc = fopen(argv[8], "r");
    int n_tok = 0, n_phr = 0;
    if (!fc || fscanf(fc, "%d %d", &n_tok, &n_phr) != 2) {
        fprintf(stderr, "cannot read %s\n", argv[8]);
        return 1;
    }
    int32_t *tokens = read_ints(fc, n_tok);
    int32_t *phrase_off = read_ints(fc, n_phr + 1);
    int32_t *sent_off = read_ints(fc, B + 1);
    fclose(fc);
    if (!tokens || !phrase_off || !sent_off) {
        fprintf(stderr, "%s is incomplete\n", argv[8]);
        return 1;
    }

    const size_t ws_bytes = dba_workspace_bytes(B, k, V, N, DBA_MAX_CONS_TOKENS);
    if (ws_bytes == 0) {
        fprintf(stderr, "shape outside the library's limits\n");
        return 1;
    }
    const size_t n_logp = (size_t)B * k * V, n_beam = (size_t)B * k;
    void *ws = NULL, *logp_dev = NULL;
    int32_t *tok_dev = NULL, *par_dev = NULL;
    float *sc_dev = NULL;
    HIP_OK(hipMalloc(&ws, ws_bytes));
    HIP_OK(hipMalloc(&logp_dev, n_logp * sizeof(float)));
    HIP_OK(hipMalloc((void **)&tok_dev, n_beam * sizeof(int32_t)));
    HIP_OK(hipMalloc((void **)&par_dev, n_beam * sizeof(int32_t)));
    HIP_OK(hipMalloc((void **)&sc_dev, n_beam * sizeof(float)));

    dba_ctx *ctx = NULL;
    if (dba_init(&ctx, B, k, V, N, eos_id, pad_id, tokens, phrase_off, sent_off, ws, ws_bytes, NULL) != DBA_OK) {
        fprintf(stderr, "dba_init: %s\n", dba_last_error(NULL));
        return 1;
    }

    FILE *fl = fopen(argv[7], "rb");
    float *logp = (float *)malloc(n_logp * sizeof(float));
    int32_t *tok = (int32_t *)malloc(n_beam * sizeof(int32_t));
    int32_t *par = (int32_t *)malloc(n_beam * sizeof(int32_t));
    float *sc = (float *)malloc(n_beam * sizeof(float));
    if (!fl || !logp || !tok || !par || !sc) {
        fprintf(stderr, "cannot open %s\n", argv[7]);
        return 1;
    }
    for (int t = 0; t < N; ++t) {
        if (fread(logp, sizeof(float), n_logp, fl) != n_logp) {
            fprintf(stderr, "%s ends before step %d\n", argv[7], t);
            return 1;
        }
        HIP_OK(hipMemcpy(logp_dev, logp, n_logp * sizeof(float), hipMemcpyHostToDevice));
        if (dba_step(ctx, (const float *)logp_dev, tok_dev, par_dev, sc_dev, NULL) != DBA_OK) {
            fprintf(stderr, "dba_step: %s\n", dba_last_error(ctx));
            return 1;
        }
        HIP_OK(hipMemcpy(tok, tok_dev, n_beam * sizeof(int32_t), hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(par, par_dev, n_beam * sizeof(int32_t), hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(sc, sc_dev, n_beam * sizeof(float), hipMemcpyDeviceToHost));
        for (int b = 0; b < B; ++b) {
            printf("step %d sent %d :", t, b);
            for (int h = 0; h < k; ++h) {
                uint32_t bits;
                memcpy(&bits, &sc[(size_t)b * k + h], 4);
                printf(" %d/%d/%08x", tok[(size_t)b * k + h], par[(size_t)b * k + h], bits);
            }
            printf("\n");
        }
    }
    fclose(fl);

    int32_t *out_tok = (int32_t *)malloc((size_t)B * N * sizeof(int32_t));
    int32_t *out_len = (int32_t *)malloc((size_t)B * sizeof(int32_t));
    int32_t *out_status = (int32_t *)malloc((size_t)B * sizeof(int32_t));
    float *out_score = (float *)malloc((size_t)B * sizeof(float));
    if (dba_finalize(ctx, out_tok, out_len, out_score, out_status) != DBA_OK) {
        fprintf(stderr, "dba_finalize: %s\n", dba_last_error(ctx));
        return 1;
    }
    for (int b = 0; b < B; ++b) {
        uint32_t bits;
        memcpy(&bits, &out_score[b], 4);
        printf("final %d : %d %d %08x :", b, out_status[b], out_len[b], bits);
        for (int i = 0; i < out_len[b] && i < N; ++i) printf(" %d", out_tok[(size_t)b * N + i]);
        printf("\n");
    }
    dba_destroy(ctx);
    HIP_OK(hipFree(ws));
    HIP_OK(hipFree(logp_dev));
    HIP_OK(hipFree(tok_dev));
    HIP_OK(hipFree(par_dev));
    HIP_OK(hipFree(sc_dev));
    return 0;
}
