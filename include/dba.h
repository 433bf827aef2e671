/*
 * libdba - the per-timestep Dynamic Beam Allocation (DBA) step of lexically
 * constrained beam search on AMD MI355X (gfx950), behind a C ABI.
 *
 * Method: Post & Vilar (2018), "Fast Lexically Constrained Decoding with
 * Dynamic Beam Allocation for Neural Machine Translation":
 *   Alg. 1  the beam-search loop this step plugs into (decoder-step -> kbest);
 *   Alg. 2  kbest-DBA: candidates from three sources, then allocate;
 *   Sec. 3.1 candidate set, constraint bookkeeping, unwinding;
 *   Sec. 3.2 bank allocation and adjustment;
 *   Sec. 3.3 finishing (no end-of-sentence before all constraints are met).
 *
 * Conventions
 *   - "host" / "device" is said for every pointer.  Device pointers are plain
 *     hipMalloc-style addresses on the current device; no framework types.
 *   - The library allocates no device memory: state, history and scratch are
 *     carved from a caller-provided workspace.
 *   - dba_step only enqueues work on the stream given at init and returns;
 *     nothing is synchronised before dba_finalize / dba_get_state.
 *   - Every function returns DBA_OK (0) or a negative code; none throws or
 *     aborts.  dba_last_error gives the text of the last failure.
 *   - One ctx is used from one host thread at a time.
 *
 * Limits (checked by dba_init): B <= 65535; 1 <= k <= 64; constraint tokens per
 * sentence <= 64; V <= 2^24; bits(k-1) + bits(V-1) + bits(Cmax) <= 32, where bits(x) is
 * the width of x and Cmax the largest constraint-token count of a sentence
 * (e.g. k = 64, 64 tokens: V <= 2^19; k = 20, 32 tokens: V <= 2^21).
 */
#ifndef DBA_H
#define DBA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DBA_API __attribute__((visibility("default")))

#define DBA_OK 0
#define DBA_EINVAL (-1) /* bad argument                                   */
#define DBA_ESTATE (-2) /* call out of order (e.g. more than N steps)     */
#define DBA_EHIP (-3)   /* a HIP runtime call failed                      */
#define DBA_ENOMEM (-4) /* workspace too small / host allocation failed   */

#define DBA_MAX_BEAM 64
#define DBA_MAX_CONS_TOKENS 64

#define DBA_FLAG_FINISHED 1 /* hypothesis has generated end-of-sentence    */
#define DBA_FLAG_DEAD 2     /* empty beam slot                             */

typedef struct dba_ctx dba_ctx;

/*
 * Bytes of device workspace dba_init needs for a job of B sentences, beam k,
 * vocabulary V and at most N steps (Alg. 1 inputs N, k).  max_cons_tokens is
 * an upper bound on the constraint tokens of any sentence (0..64).
 * Returns 0 if an argument is out of range.
 */
DBA_API size_t dba_workspace_bytes(int B, int k, int V, int N, int max_cons_tokens);

/*
 * decoder-init of Alg. 1 plus the constraints of every sentence (Sec. 3:
 * word and phrasal constraints; C = total tokens).
 *
 *   out              host: receives the new ctx (host object, free with dba_destroy)
 *   B, k, V, N       batch, beam size, target vocabulary size, max output length
 *   eos_id, pad_id   end-of-sentence id; id written into empty slots and used
 *                    as the sole continuation of finished hypotheses
 *   cons_tokens      host [total tokens]   all constraint token ids, phrase after phrase
 *   phrase_offsets   host [total phrases+1] phrase p = cons_tokens[phrase_offsets[p] .. phrase_offsets[p+1])
 *   sent_offsets     host [B+1]            sentence b owns phrases sent_offsets[b] .. sent_offsets[b+1]
 *                    (a sentence may have none).  The three arrays are copied; the caller may free them.
 *   workspace_dev    device, 256-byte aligned, >= dba_workspace_bytes(...) bytes; owned by the
 *                    caller, must stay valid and untouched until dba_destroy
 *   hip_stream       a hipStream_t (NULL = default stream); all work of this ctx is enqueued on it
 *
 * The initial beam of every sentence is one live, empty hypothesis in slot 0
 * with score +0.0; the other k-1 slots are empty.
 * Errors: DBA_EINVAL for sizes < 1, B > 65535, k > 64, k > V, ids outside [0,V),
 * eos_id == pad_id, a constraint token equal to eos_id or pad_id, an empty
 * phrase, offsets not starting at 0 / not non-decreasing, more than 64 tokens
 * in a sentence, the width limit above, a misaligned workspace;
 * DBA_ENOMEM if workspace_bytes is too small; DBA_EHIP on a runtime failure.
 */
DBA_API int dba_init(dba_ctx **out, int B, int k, int V, int N, int eos_id, int pad_id,
             const int32_t *cons_tokens, const int32_t *phrase_offsets,
             const int32_t *sent_offsets, void *workspace_dev, size_t workspace_bytes,
             void *hip_stream);

/*
 * One call of kbest-DBA (Alg. 2) for all B sentences.
 *
 *   logp_dev        device [B,k,V] fp32, row-major, 4-byte aligned, read only; row h of
 *                   sentence b holds the log-probabilities of extending the hypothesis in
 *                   beam slot h of the previous step's output (the "scores" matrix of
 *                   Sec. 2 before the hypothesis score is added).  An entry of -inf is legal
 *                   (that extension does not exist); NaN and +inf are not.  The content of
 *                   rows of empty slots is ignored, but the whole [B,k,V] extent must be
 *                   readable.  Must stay valid until the stream has passed this step.
 *   out_token_dev   device [B,k] int32: token of each new beam slot, best first (pad_id if empty)
 *   out_backptr_dev device [B,k] int32: beam slot of the parent hypothesis (-1 if empty)
 *   out_score_dev   device [B,k] fp32 : cumulative score = parent score + logp, one fp32 add
 *                   (-inf if empty)
 *   out_flags_dev   device [B,k] uint8: DBA_FLAG_* bits; may be NULL
 *
 * Under DBA_OPT_NORMALIZE_FINISHED / DBA_OPT_PRUNE_THRESHOLD the scores and the occupied slots
 * are as described at dba_set_option.  Any of the first three outputs may also be NULL (the beam
 * is kept inside the ctx anyway).  Asynchronous.  Errors: DBA_EINVAL (NULL ctx / logp), DBA_ESTATE
 * after N steps, DBA_EHIP if the launch fails.
 */
DBA_API int dba_step(dba_ctx *ctx, const float *logp_dev, int32_t *out_token_dev,
             int32_t *out_backptr_dev, float *out_score_dev, uint8_t *out_flags_dev);

/*
 * dba_step for a decoder that hands over its log-probs in another element type.  logp_dev is
 * device [B,k,V] of that type, row-major, aligned to the element size (rows need no further
 * alignment).  A 16-bit log-prob is widened to fp32 exactly (both conversions are exact) and the
 * score is then the same single fp32 addition parent score + logp; everything else is dba_step.
 * The formats may change from call to call.  DBA_EINVAL for an unknown format.
 */
#define DBA_LOGP_F32 0  /* fp32 (what dba_step takes)   */
#define DBA_LOGP_F16 1  /* IEEE binary16                */
#define DBA_LOGP_BF16 2 /* bfloat16                     */
DBA_API int dba_step_fmt(dba_ctx *ctx, const void *logp_dev, int logp_format, int32_t *out_token_dev,
                         int32_t *out_backptr_dev, float *out_score_dev, uint8_t *out_flags_dev);

/*
 * dba_step_fmt for callers that must not allocate and want the library to bring its own scratch:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  (No entry
 * point of this library allocates device memory; here even the scratch that passes a step's
 * intermediate results - every beam row's list of best sums and its constraint-token keys - from
 * the first launch to the second is not taken from the caller's workspace but from a fixed array
 * inside the library, 8 MiB per GPU, resolved once per device.)  Same arguments, same results and
 * the same asynchronous behaviour as dba_step_fmt; calls may be mixed with dba_step / dba_step_fmt
 * on the same ctx from step to step.  Nothing in the array has to start at zero: every step
 * overwrites what it reads.
 * Limits: B*k <= DBA_NOALLOC_MAX_ROWS, else DBA_EINVAL with a message (no launch).  All contexts on
 * one GPU share that GPU's array: steps of different contexts that overlap in time (different
 * streams) race on it - keep such steps on one stream or use dba_step.  The device that was current
 * at dba_init must be current.  Calls no hipMalloc / hipFree.
 */
#define DBA_NOALLOC_MAX_ROWS 8192
DBA_API int dba_step_noalloc(dba_ctx *ctx, const void *logp_dev, int logp_format, int32_t *out_token_dev,
                             int32_t *out_backptr_dev, float *out_score_dev, uint8_t *out_flags_dev);

/*
 * End of Alg. 1 with Sec. 3.3 and the length normalisation of Sec. 4: for each
 * sentence the completed hypothesis (end-of-sentence generated, hence all
 * constraints met) with the best score/length, traced back through the
 * recorded steps.  Only the final beam is searched unless
 * DBA_OPT_TRACK_COMPLETED is set (a completed hypothesis can lose its slot to
 * better-scoring candidates of the topmost bank).  Synchronises the stream.
 *
 *   out_tokens_host host [B,N] int32, pad_id-filled beyond the length
 *   out_len_host    host [B]   int32, tokens incl. end-of-sentence
 *   out_score_host  host [B]   fp32, score of the returned hypothesis as the beam holds it
 *                   (cumulative; per word under DBA_OPT_NORMALIZE_FINISHED)
 *   out_status_host host [B]   int32, 1 = a completed hypothesis was found; 0 = none (the
 *                   returned one is then the live slot with most constraints met,
 *                   then best score)
 * May be called after any number of steps, more than once.
 */
DBA_API int dba_finalize(dba_ctx *ctx, int32_t *out_tokens_host, int32_t *out_len_host,
                 float *out_score_host, int32_t *out_status_host);

/*
 * Copy the current beam state to the host (synchronises the stream).  Every
 * pointer is host [B,k] and may be NULL.  met_mask bit i = constraint token i
 * of the sentence (in the order given to dba_init) is marked met (Sec. 3.1);
 * inprog_phrase = index within the sentence of the phrase under way (-1 none),
 * inprog_pos = how many of its tokens are met.
 */
DBA_API int dba_get_state(dba_ctx *ctx, float *score_host, uint64_t *met_mask_host,
                  int32_t *inprog_phrase_host, int32_t *inprog_pos_host, int32_t *length_host,
                  uint8_t *flags_host);

/*
 * Options, settable between dba_init and the first dba_step (DBA_ESTATE afterwards,
 * DBA_EINVAL for an unknown option or a NaN value).  The defaults give the bare
 * algorithm of Alg. 2; the others are the settings of the paper's experiments.
 *   DBA_OPT_ADJUSTMENT          1 (default): bank sizes are adjusted as in Sec. 3.2; 0: they stay
 *                               at the base split and a bank that cannot fill its slots leaves
 *                               them empty - with k = b(C+1) the grid-beam-search simulation of
 *                               Sec. 5.
 *   DBA_OPT_NORMALIZE_FINISHED  0 (default): the beam holds cumulative scores and dba_finalize
 *                               divides by the length; non-zero: a hypothesis that generates
 *                               end-of-sentence is stored with score / length (one fp32 division,
 *                               the length counts end-of-sentence) from that step on, as in
 *                               Sec. 4 and the caption of Fig. 9; inside the step in which it
 *                               completes it still competes with its cumulative score, and
 *                               dba_finalize ranks completed hypotheses by the stored score.
 *   DBA_OPT_PRUNE_THRESHOLD     negative (default): no pruning; t >= 0: after every step, each
 *                               hypothesis, completed or not, whose stored score is below
 *                               (best stored score of a completed hypothesis on the new beam) - t
 *                               is removed and the others close ranks (Sec. 4, Sec. 6.3; the
 *                               paper uses 20).  The value is rounded to fp32; the difference is
 *                               one fp32 subtraction and a score equal to it survives.
 *   DBA_OPT_TRACK_COMPLETED     0 (default): dba_finalize searches the final beam only, so a completed
 *                               hypothesis that lost its slot meanwhile (it sits in the topmost bank
 *                               and candidates with higher scores can take its place) is forgotten;
 *                               non-zero: every step remembers, per sentence, the best completed
 *                               hypothesis seen on any beam so far - ranked by score per word, a tie
 *                               keeps the earliest step, then the lowest slot - and dba_finalize
 *                               returns it (Sec. 3.3: the answer is the best-scoring finished hypothesis).
 *   DBA_OPT_MERGE_WAVES         0 (default), 4 or 8 (anything else: DBA_EINVAL): wavefronts of the
 *                               workgroup that handles one sentence in the second launch of a step.
 *                               The results are the same for every setting; only the time differs.
 *                               0 lets the library choose for the shortest step of a single decode
 *                               (four up to k = 16, eight beyond).  Four-wave workgroups are placed more
 *                               easily on a GPU that is busy with other work: the better setting where
 *                               several decodes are in flight on the same GPU.
 */
#define DBA_OPT_ADJUSTMENT 2
#define DBA_OPT_NORMALIZE_FINISHED 3
#define DBA_OPT_PRUNE_THRESHOLD 4
#define DBA_OPT_TRACK_COMPLETED 5
#define DBA_OPT_MERGE_WAVES 6
DBA_API int dba_set_option(dba_ctx *ctx, int option, double value);

/*
 * The stopping tests (synchronises the stream): all_finished_host, host [B] uint8, receives for
 * every sentence DBA_STOP_ALL (bit 0) when its beam is not empty and holds completed hypotheses
 * only - Sec. 4: decoding stops, further steps would only carry them along - and DBA_STOP_ANY
 * (bit 1) when at least one hypothesis on the beam is completed - the early stopping that
 * Sec. 6.3 mentions as the alternative to pruning.  0 before the first step.
 */
#define DBA_STOP_ALL 1
#define DBA_STOP_ANY 2
DBA_API int dba_get_finished(dba_ctx *ctx, uint8_t *all_finished_host);

/* Number of dba_step calls made so far (or DBA_EINVAL). */
DBA_API int dba_steps_done(const dba_ctx *ctx);

/* Frees the host-side ctx only; device memory belongs to the caller. */
DBA_API void dba_destroy(dba_ctx *ctx);

/* Text of the last error on this ctx, or of the last failed dba_init of the
 * calling thread if ctx is NULL.  Never NULL. */
DBA_API const char *dba_last_error(const dba_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DBA_H */
