// Device side of the DBA step (Post & Vilar 2018, Alg. 2, Sec. 3.1-3.3) for gfx950.
//
// Two phases per step:
//   stream phase  one workgroup per beam row (b,h): a single pass over the V
//                 log-probs of that row - score add, end-of-sentence mask,
//                 exact top-k of the row (which holds the row's best token
//                 and its share of the sentence's top-k) written as one sorted
//                 64-key list per row - plus the row's expandable constraint
//                 tokens (Alg. 2 inner loop): which they are and their sums;
//                 every key of either kind carries the bank it would land in
//                 (the constraints met after add(), Sec. 3.1): selection keys;
//   merge phase   one workgroup per sentence: the bar of the sentence's top-k
//                 from the row lists, dedup, bank counts, allocation with
//                 adjustment, selection, the state transition add() in full
//                 for the winners, new beam.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "wave_topk.hpp"

namespace dba {

constexpr int kMaxBeam = 64;
constexpr int kMaxCons = 64;          // constraint tokens (and phrases) per sentence
constexpr int kBlock = 256;           // threads per workgroup of the small helper kernels
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kStreamWaves = 8;       // most waves a stream-phase workgroup (one beam row) can have: 4 or 8 are used
constexpr int kTileLoads = 4;         // 16-byte loads per lane and tile in the stream phase
constexpr int kFmtF32 = 0;            // element type of the log-probs: fp32,
constexpr int kFmtF16 = 1;            // IEEE binary16,
constexpr int kFmtBF16 = 2;           // bfloat16 (the 16-bit types are widened exactly; the sum is fp32)
constexpr int kFinFinished = 1;       // beam-state flag: the hypothesis has generated end-of-sentence
constexpr int kFinEosBlocked = 4;     // beam-state flag: constraints unmet, end-of-sentence not allowed (Sec. 3.3)

struct StepParams {
    int B, k, V;
    int eos_id, pad_id;
    int met_bits;                     // width of the bank field in the packed selection key
    int tok_bits;                     // width of the token field of a coordinate: (h << tok_bits) | w
    int first_step;                   // 1: the beam is the initial one (only slot 0 of a sentence is live)
    int cand_cap;                     // candidate keys the merge phase's dynamic LDS holds (a multiple of 64)
    int adjust;                       // 0: bank sizes stay at the base split (Sec. 5)
    int normalize;                    // 1: a hypothesis completing now is stored with sum / length (Sec. 4)
    float prune;                      // >= 0: threshold pruning against the best completed hypothesis (Sec. 4)
    int track;                        // 1: keep a record of the best completed hypothesis seen on any beam (Sec. 3.3)
    int step;                         // index of this step, from 0
    const void *logp;                 // [B,k,V] in the element type the kernel is instantiated for
    // beam before the step
    const float *score_cur;           // [B,k]  (-inf: empty slot)
    const u64 *met_cur;               // [B,k]  bit i = constraint token i met
    const int32_t *ipq_cur;           // [B,k]  phrase under way * 256 + tokens met in it, or -1
    const int32_t *len_cur;           // [B,k]
    const uint8_t *fin_cur;           // [B,k]  kFin* flags
    const u64 *inc_cur;               // [B,k]  bit j = phrase j is not complete
    const int32_t *nxt_cur;           // [B,k]  next token of the phrase under way (-1: none)
    // beam after the step
    float *score_nxt;
    u64 *met_nxt;
    int32_t *ipq_nxt;
    int32_t *len_nxt;
    uint8_t *fin_nxt;
    u64 *inc_nxt;
    int32_t *nxt_nxt;
    // constraints
    const int32_t *cons_tok;          // [B,64]
    const int32_t *phr_off;           // [B,65] token offset of each phrase, phr_off[b][P] = C
    const int32_t *nphr;              // [B]
    const int32_t *first_tok;         // [B,64] first token of phrase j
    const u64 *same_first_lower;      // [B,64] phrase j: the lower phrases with the same first token
    const u64 *first_bucket;          // [B,64] bucket w & 63: the phrases whose first token has these low six bits
    const int32_t *bucket_tok;        // [B,64] that first token if the bucket's phrases agree on it; -1 none, -2 they differ
    // scratch
    u64 *rowlists;                    // [B*k,64] every row's best sums, decreasing, as selection-key bodies
    u64 *conskeys;                    // [B*k,64] selection keys (bank, score image, ~flat) of the
                                      //          row's expandable constraint tokens, 0 = none
    // outputs (each may be null)
    int32_t *out_token, *out_backptr;
    float *out_score;
    uint8_t *out_flags;
    int32_t *hist_token, *hist_backptr;   // row t of the history, [B,k]
    uint8_t *all_finished;            // [B] bit 0: the new beam is not empty and every hypothesis on it is completed;
                                      //     bit 1: some hypothesis on it is completed
    struct BestCompleted *best;       // [B] the record kept under `track`
};

// The best completed hypothesis a sentence has had on any of its beams so far (Sec. 3.3: the answer is
// the best-scoring finished hypothesis; Sec. 4 ranks completed hypotheses by score per word).
struct __attribute__((aligned(32))) BestCompleted {
    int have;          // 0: nothing completed yet
    int step, slot;    // where it was first seen: the beam after step `step`, place `slot`
    int len;           // its length, end-of-sentence included
    float q;           // its score per word
    float score;       // its score as that beam held it
    int pad[2];
};

// constraints of one sentence: token ids phrase after phrase, phrase p = tok[poff[p] .. poff[p+1])
struct ConsTab {
    int tok[kMaxCons];
    int poff[kMaxCons + 1];
};

// one hypothesis of the beam before the step, as the merge phase keeps it in LDS (two 16-byte reads)
struct __attribute__((aligned(16))) HypState {
    u64 met;       // bit i = constraint token i met
    u64 inc;       // bit j = phrase j not complete
    int ipq;       // phrase under way * 256 + tokens met in it, or -1
    int nxt;       // next token of the phrase under way (-1: none under way)
    int len;
    int misc;      // finished flag | constraints met << 8
};

constexpr int kMergeWavesMax = 8;     // most waves a merge-phase workgroup (one sentence) can have: 4 or 8 are used

struct MergeSmem {
    uint32_t ws[kMergeWavesMax][kWave];      // every wave's best score images
    uint32_t wf[kMergeWavesMax][kWave];      // and the greatest images its merges dropped
    uint32_t ws2[kMergeWavesMax][kWave];     // every wave's best low words among tied keys
    HypState hyp[kMaxBeam];
    u64 sel[kMaxBeam];
    int slot[kMaxBeam];               // place in the new beam of the selected key i
    ConsTab ct;
    u64 fbucket[kMaxCons];            // phrases by the low six bits of their first token
    int btok[kMaxCons];               // and that token where a bucket's phrases agree on it (-1 none, -2 they differ)
    // per bank (constraints met, 0..64); sized for every value the 7-bit bank field of a key can hold
    int cnt[2 * kMaxCons];
    int alloc[2 * kMaxCons];
    int start[2 * kMaxCons];
    uint32_t bar_score;               // with eight waves: the score image of the bar of the k best, from the waves that join the lists,
    int bar_need;                     // and the places left for keys that tie at that score (-1: no tie to settle)
    int ncand;
    int nsel;
    u64 kept;                         // pruning: bit i = the hypothesis at place i of the new beam stays
};

// ---------------------------------------------------------------------------
// stream phase
// ---------------------------------------------------------------------------
struct RowTop {
    u64 list;      // this lane's entry of the wave's decreasing top-64
    u64 kth;       // key at place k-1 (0 while fewer than k entries)
    float floor;   // a proven lower bound of the row's k-th best sum (-inf if none)
    float thr;     // sums below this cannot reach the row's top k; never below -FLT_MAX, so
                   // that "s >= thr" also rejects -inf sums
};

constexpr float kLowestFinite = -3.402823466e+38f;

__device__ __forceinline__ void refresh_threshold(RowTop &st, int kk)
{
    st.kth = read_lane(st.list, kk - 1);
    const float own = (st.kth == 0) ? kLowestFinite : float_from_ord((uint32_t)(st.kth >> 32));
    st.thr = fmaxf(fmaxf(st.floor, own), kLowestFinite);
}

// Key of a wave-uniform element, built from uniform values (scalar unit).
__device__ __forceinline__ u64 make_key_uniform(uint32_t sbits, uint32_t flat)
{
    if (sbits == 0x80000000u) sbits = 0;                       // -0.0 -> +0.0
    const uint32_t mask = (uint32_t)((int32_t)sbits >> 31);    // all ones for negative floats
    const uint32_t ord = sbits ^ (mask | 0x80000000u);
    return ((u64)ord << 32) | (u64)(0xFFFFFFFFu - flat);
}

constexpr int kStageCap = 128;        // candidate keys one wave can park in LDS between flushes

// Candidates of one wave are parked in LDS (stage[0..cnt)) and folded into the wave's sorted
// list 64 at a time: one 64-lane sort and one merge per chunk instead of one serial insert per
// candidate.  The threshold tightens at every flush.
__device__ __attribute__((noinline)) u64 fold_stage(u64 list, const u64 *stage, int cnt)
{
    const int lane = lane_id();
    for (int base = 0; base < cnt; base += kWave) {
        const u64 key = (base + lane < cnt) ? stage[base + lane] : 0ull;
        list = merge_desc<u64>(list, sort64_desc<u64>(key));
    }
    return list;
}

__device__ __forceinline__ void flush_stage(RowTop &st, u64 *stage, int &cnt, int kk)
{
    st.list = fold_stage(st.list, stage, cnt);
    cnt = 0;
    refresh_threshold(st, kk);
}

// Wave-wide: every lane offers one element; m = ballot of the lanes whose sum may belong to
// the row's top k (m != 0).  Lane l's coordinate is flat0 + l*lane_stride.
__device__ __forceinline__ void stage_candidates(RowTop &st, u64 *stage, int &cnt, float s, u64 m,
                                                 uint32_t flat0, uint32_t lane_stride, int kk)
{
    const int n = __popcll(m);
    if (cnt + n > kStageCap) flush_stage(st, stage, cnt, kk);
    const int lane = lane_id();
    const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    if ((m >> lane) & 1ull) stage[pos] = make_key(s, flat0 + (uint32_t)lane * lane_stride);
    cnt += n;
}

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// max of four finite-or-infinite floats in two instructions (the inputs are never NaN, so the
// quieting moves a generic fmaxf would add are not needed)
__device__ __forceinline__ float max4(const v4f &x)
{
    float t, m;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(t) : "v"(x.x), "v"(x.y), "v"(x.z));
    asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(t), "v"(x.w));
    return m;
}

// ---- element formats of the log-prob tensor ----------------------------------------------
// A lane reads 16 bytes at a time: a "group" of G consecutive elements.  Every format answers
// three questions about a group: may any of its elements reach the threshold (cheap, and
// allowed to say yes too often, never no wrongly), what are its G elements as fp32 (exact), and
// which single fp32 value is certainly not above the group's greatest element (for the
// threshold floor).  The sum itself is always one fp32 addition prev + element.
template <int FMT>
struct Logp;

template <>
struct Logp<kFmtF32> {
    static constexpr int G = 4;
    typedef float elem_t;
    typedef v4f vec_t;
    struct Quick {};                                  // the quick test uses the fp32 threshold itself
    static __device__ __forceinline__ vec_t neg_inf() { return v4f{-INFINITY, -INFINITY, -INFINITY, -INFINITY}; }
    static __device__ __forceinline__ Quick quick(float, float) { return Quick{}; }
    // rounding is monotone, so max(prev + x_i) == prev + max(x_i): one add decides for four
    static __device__ __forceinline__ bool may_reach(const vec_t &x, float prev, float thr, const Quick &)
    {
        return prev + max4(x) >= thr;
    }
    static __device__ __forceinline__ void widen(const vec_t &x, float (&f)[G])
    {
        f[0] = x.x;
        f[1] = x.y;
        f[2] = x.z;
        f[3] = x.w;
    }
    static __device__ __forceinline__ float some_element_at_most_max(const vec_t &x) { return max4(x); }
    static __device__ __forceinline__ void drop(vec_t &x, int c)
    {
        if (c == 0) x.x = -INFINITY;
        if (c == 1) x.y = -INFINITY;
        if (c == 2) x.z = -INFINITY;
        if (c == 3) x.w = -INFINITY;
    }
    static __device__ __forceinline__ float widen_one(elem_t e) { return e; }
};

// The two 16-bit formats are sign-magnitude like fp32, so among negative values a greater bit
// pattern is a smaller number, and every non-negative pattern is below every negative one:
// "element >= bound" for a negative bound is "pattern <= pattern of the bound" on unsigned
// 16-bit integers.  The quick test therefore needs no conversion at all: the unsigned minimum
// of the group's eight patterns (packed 16-bit minima) against one precomputed pattern.
template <int FMT>
struct Logp16 {
    static constexpr int G = 8;
    typedef uint16_t elem_t;
    typedef v4u vec_t;
    static constexpr uint32_t kNegInf = FMT == kFmtF16 ? 0xFC00u : 0xFF80u;
    struct Quick {
        uint32_t umax;    // greatest pattern whose sum still reaches the threshold (0xFFFF: test everything)
    };
    static __device__ __forceinline__ vec_t neg_inf()
    {
        const uint32_t w = kNegInf | (kNegInf << 16);
        return v4u{w, w, w, w};
    }
    static __device__ __forceinline__ float widen_bits(uint32_t h)
    {
        if constexpr (FMT == kFmtBF16) return __uint_as_float(h << 16);
        else return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
    }
    static __device__ __forceinline__ float widen_one(elem_t e) { return widen_bits(e); }
    // round-to-nearest pattern of a negative finite fp32 (a starting point only: quick() corrects it)
    static __device__ __forceinline__ uint32_t narrow_bits(float d)
    {
        if constexpr (FMT == kFmtBF16) {
            const uint32_t u = __float_as_uint(d);
            return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
        } else {
            return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)d);
        }
    }
    // umax = the pattern of the smallest element x with fp32(prev + x) >= thr, found exactly: a
    // rounded guess, then single steps while the next smaller element still reaches thr, then
    // single steps back while the element itself does not.  If the steps run out on the way
    // down, everything is tested (never wrong, only slower).  thr never decreases, so a value
    // computed for an older thr stays valid.
    static __device__ __forceinline__ Quick quick(float prev, float thr)
    {
        const float d = thr - prev;
        if (!(d < 0.0f)) return Quick{0xFFFFu};
        uint32_t u = narrow_bits(d);
        if (u < 0x8000u) u = 0x8000u;
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (prev + widen_bits(u + 1u) >= thr) ++u;
        if (prev + widen_bits(u + 1u) >= thr) return Quick{0xFFFFu};
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (u >= 0x8000u && !(prev + widen_bits(u) >= thr)) --u;
        return Quick{u};
    }
    // unsigned minimum of the two 16-bit halves, both halves at once
    static __device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b)
    {
        uint32_t r;
        asm("v_pk_min_u16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
        return r;
    }
    static __device__ __forceinline__ uint32_t min_pattern(const vec_t &x)
    {
        const uint32_t c = pk_min_u16(pk_min_u16(x.x, x.y), pk_min_u16(x.z, x.w));
        return min(c & 0xFFFFu, c >> 16);
    }
    static __device__ __forceinline__ bool may_reach(const vec_t &x, float, float, const Quick &q)
    {
        return min_pattern(x) <= q.umax;
    }
    static __device__ __forceinline__ void widen(const vec_t &x, float (&f)[G])
    {
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = widen_bits(w[i] & 0xFFFFu);
            f[2 * i + 1] = widen_bits(w[i] >> 16);
        }
    }
    // the element with the smallest pattern: the greatest one if none is positive, else some
    // positive one - in both cases an element of the group
    static __device__ __forceinline__ float some_element_at_most_max(const vec_t &x)
    {
        return widen_bits(min_pattern(x));
    }
    static __device__ __forceinline__ void drop(vec_t &x, int c)
    {
        const uint32_t keep = (c & 1) ? 0x0000FFFFu : 0xFFFF0000u;
        const uint32_t put = (c & 1) ? (kNegInf << 16) : kNegInf;
        if ((c >> 1) == 0) x.x = (x.x & keep) | put;
        if ((c >> 1) == 1) x.y = (x.y & keep) | put;
        if ((c >> 1) == 2) x.z = (x.z & keep) | put;
        if ((c >> 1) == 3) x.w = (x.w & keep) | put;
    }
};
template <>
struct Logp<kFmtF16> : Logp16<kFmtF16> {};
template <>
struct Logp<kFmtBF16> : Logp16<kFmtBF16> {};

// The log-probs are read exactly once: non-temporal loads keep them from displacing
// anything useful in the caches.  nv = groups in the row's aligned body.
template <int U, typename VEC>
__device__ __forceinline__ void load_tile(const VEC *__restrict__ vec, int nv, int tile, int lane, VEC (&x)[U],
                                          const VEC fill)
{
    const int base = tile * (kWave * U);
    if (base + kWave * U <= nv) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = __builtin_nontemporal_load(vec + base + u * kWave + lane);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = base + u * kWave + lane;
            x[u] = (i < nv) ? __builtin_nontemporal_load(vec + i) : fill;
        }
    }
}

// Sec. 3.3: while constraints are unmet the end-of-sentence entry does not exist.  rel = its
// position inside the tile in elements (wave-uniform); the one lane holding it drops it.
template <int U, int FMT>
__device__ __forceinline__ void block_eos(typename Logp<FMT>::vec_t (&x)[U], int rel, int lane)
{
    constexpr int G = Logp<FMT>::G;
    const int uu = rel / (G * kWave), ln = (rel / G) & (kWave - 1), c = rel & (G - 1);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (u == uu && lane == ln) Logp<FMT>::drop(x[u], c);
}

// LDS shared by the waves of one row's workgroup during the stream phase.
struct StreamSmem {
    u64 wl[kStreamWaves][kWave];        // the waves' lists, for the final merge
    u64 stage[kStreamWaves][kStageCap]; // candidates parked between flushes
    uint32_t boot[kStreamWaves][kWave]; // sorted per-lane maxima of every wave's first tile (order images)
    int parked[kStreamWaves];           // end of the row: keys each wave has left in its stage,
    int has_list[kStreamWaves];         // and whether it holds a list from earlier folds
};

// One wave's share of one row: tiles wave, wave+nwaves, ... of 64*U groups of 16 bytes each.
// Must be called by every thread of the workgroup (it contains one barrier).
//
// s = prev + logp is a single fp32 add (a 16-bit log-prob is widened exactly first).  An
// element is looked at closely only if its sum can still reach the row's k best (>=: a later
// element may tie the k-th score and win on the coordinate); Logp<FMT>::may_reach decides that
// for a whole 16-byte group at once.
//
// Thresholds.  (1) Every lane takes an element of its share of the wave's first two tiles (the
// greatest, where the format finds it cheaply); the k-th greatest of all the workgroup's
// per-lane values is a floor: k different lanes hold an element at least that large, so nothing
// below it can be among the row's k best.  (2) A wave whose stage fills up folds it into its
// list; from then on the score of the list's k-th entry bounds its share of the row.  With the
// floor in place that is rare: a wave parks about k keys per row.  The row's best element is
// never below any bound, so it always survives.
template <int U, int FMT>
struct RowStream {
    typedef Logp<FMT> F;
    typedef typename F::vec_t vec_t;
    typedef typename F::elem_t elem_t;
    static constexpr int G = F::G;

    const elem_t *row;
    const vec_t *vec;
    int V, head, nv, tail, ntiles;
    vec_t cur[U], nxt[U];

    // Issues the loads of this wave's first two tiles.  Needs nothing of the hypothesis, so it
    // runs before the beam state has arrived.
    __device__ __forceinline__ void begin(const elem_t *__restrict__ row_, int V_, int wave, int nwaves)
    {
        const int lane = lane_id();
        row = row_;
        V = V_;
        const uintptr_t addr = reinterpret_cast<uintptr_t>(row);
        head = (int)(((16u - (unsigned)(addr & 15u)) & 15u) / (unsigned)sizeof(elem_t));
        if (head > V) head = V;
        nv = (V - head) / G;
        tail = V - head - nv * G;
        vec = reinterpret_cast<const vec_t *>(row + head);
        ntiles = (nv + kWave * U - 1) / (kWave * U);
#pragma unroll
        for (int u = 0; u < U; ++u) nxt[u] = F::neg_inf();
        if (wave < ntiles) load_tile<U>(vec, nv, wave, lane, cur, F::neg_inf());
        if (wave + nwaves < ntiles) load_tile<U>(vec, nv, wave + nwaves, lane, nxt, F::neg_inf());
    }

    // Returns the number of keys left parked in sm.stage[wave] (not yet folded into st.list).
    __device__ __forceinline__ int run(float prev, int eos_block, uint32_t flat_base, int kk, int wave,
                                       int nwaves, StreamSmem &sm, RowTop &st);
};

template <int U, int FMT>
__device__ __forceinline__ int RowStream<U, FMT>::run(float prev, int eos_block, uint32_t flat_base, int kk,
                                                      int wave, int nwaves, StreamSmem &sm, RowTop &st)
{
    const int lane = lane_id();
    constexpr int kTileElems = G * kWave * U;
    const int eos_rel0 = eos_block >= 0 ? eos_block - head : -1;   // position in the aligned body
    int tl = wave;
    uint32_t boot = ord_from_float(-INFINITY);
    if (tl < ntiles) {
        // both tiles already requested take part in the floor (8 KB per wave, 32 KB per row)
        const int rel = eos_rel0 - tl * kTileElems;
        if (eos_rel0 >= 0 && rel >= 0 && rel < kTileElems) block_eos<U, FMT>(cur, rel, lane);
        float lane_max = F::some_element_at_most_max(cur[0]);
#pragma unroll
        for (int u = 1; u < U; ++u) {
            const float mu = F::some_element_at_most_max(cur[u]);
            asm("v_max_f32 %0, %1, %2" : "=v"(lane_max) : "v"(lane_max), "v"(mu));
        }
        if (tl + nwaves < ntiles) {
            const int rel2 = eos_rel0 - (tl + nwaves) * kTileElems;
            if (eos_rel0 >= 0 && rel2 >= 0 && rel2 < kTileElems) block_eos<U, FMT>(nxt, rel2, lane);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float mu = F::some_element_at_most_max(nxt[u]);
                asm("v_max_f32 %0, %1, %2" : "=v"(lane_max) : "v"(lane_max), "v"(mu));
            }
        }
        boot = sort64_desc<uint32_t>(ord_from_float(prev + lane_max));
    }
    if (nwaves > 1) {
        sm.boot[wave][lane] = boot;
        __syncthreads();
        const int share = kWave / nwaves;              // entries of every wave's list that fit one 64-lane sort
        if (kk <= 3 * share) {
            // Any k values that different lanes hold give a valid floor, so the best `share` of every
            // wave's list, sorted once, do: the k-th of them is the k-th of all unless one wave
            // holds more than `share` of the k greatest (then it is a little lower, never wrong).
            boot = sort64_desc<uint32_t>(sm.boot[lane / share][lane % share]);
        } else {
            for (int w = 0; w < nwaves; ++w)
                if (w != wave) boot = merge_desc<uint32_t>(boot, sm.boot[w][lane]);
        }
    }
    st.floor = float_from_ord((uint32_t)__builtin_amdgcn_readlane((int)boot, kk - 1));
    st.thr = fmaxf(st.floor, kLowestFinite);
    typename F::Quick quick = F::quick(prev, st.thr);
    u64 *stage = sm.stage[wave];
    int cnt = 0;
    // one tile: test its U groups, park what may belong to the top k
    auto examine = [&](const vec_t (&t)[U], int tile) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const vec_t x = t[u];
            if (__any(F::may_reach(x, prev, st.thr, quick))) {
                const uint32_t flat0 = flat_base + (uint32_t)(head + G * ((tile * U + u) * kWave));
                float f[G];
                F::widen(x, f);
#pragma unroll
                for (int c = 0; c < G; ++c) {
                    const float sc = prev + f[c];
                    const u64 mc = __ballot(sc >= st.thr);
                    if (mc) stage_candidates(st, stage, cnt, sc, mc, flat0 + (uint32_t)c, (uint32_t)G, kk);
                }
            }
        }
    };
    // after a tile: start the load that refills its registers (two tiles ahead) and make the
    // other buffer ready (end-of-sentence mask, the quick test's form of the threshold)
    auto advance = [&](vec_t (&done)[U], vec_t (&next)[U], int next_tile) {
        if (next_tile + nwaves < ntiles) load_tile<U>(vec, nv, next_tile + nwaves, lane, done, F::neg_inf());
        if (next_tile < ntiles) {
            const int rel = eos_rel0 - next_tile * kTileElems;
            if (eos_rel0 >= 0 && rel >= 0 && rel < kTileElems) block_eos<U, FMT>(next, rel, lane);
            quick = F::quick(prev, st.thr);
        }
    };
    while (tl < ntiles) {
        examine(cur, tl);
        advance(cur, nxt, tl + nwaves);
        tl += nwaves;
        if (tl >= ntiles) break;
        examine(nxt, tl);
        advance(nxt, cur, tl + nwaves);
        tl += nwaves;
    }
    // elements before the first / after the last 16-byte aligned group (rows whose length or
    // start is not a multiple of one group): fewer than two groups, one element per lane
    if (wave == 0 && head + tail > 0) {
        const bool mine = lane < head + tail;
        const int w = lane < head ? lane : head + nv * G + (lane - head);
        const float s = mine ? prev + F::widen_one(row[w]) : -INFINITY;
        u64 m = __ballot(mine && (s >= st.thr) && (w != eos_block));
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const int wl = l < head ? l : head + nv * G + (l - head);
            const uint32_t sbits = (uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(s), l);
            if (cnt + 1 > kStageCap) flush_stage(st, stage, cnt, kk);
            if (lane == 0) stage[cnt] = make_key_uniform(sbits, flat_base + (uint32_t)wl);
            cnt += 1;
        }
    }
    return cnt;
}

// End of a row.  Each wave arrives with a sorted list from earlier folds (usually none: with
// the floor in place a wave parks a few dozen keys per row and never fills its stage) and the
// keys still parked in its stage.  The parked keys of all waves are pooled and sorted in chunks
// of 64 - one chunk in the common case, sorted by one wave - instead of one sort per wave plus
// a merge per wave.  The wave that finishes the row (fin_wave) rotates with the row index, so
// that the rows sharing a compute unit finish on different SIMDs.  Returns the row's list to
// the lanes of fin_wave.  Called by every thread of the workgroup (one or two barriers).
__device__ __forceinline__ u64 finish_row(StreamSmem &sm, u64 list, int parked, int wave, int nwaves,
                                          int fin_wave)
{
    const int lane = lane_id();
    const bool mine_has = read_lane(list, 0) != 0;
    if (lane == 0) {
        sm.parked[wave] = parked;
        sm.has_list[wave] = mine_has ? 1 : 0;
    }
    __syncthreads();
    // keys parked by waves 0..w-1 (pre[w]); all of them (n)
    int pre[kStreamWaves + 1];
    int any = 0;
    pre[0] = 0;
#pragma unroll
    for (int w = 0; w < kStreamWaves; ++w) {
        pre[w + 1] = pre[w] + (w < nwaves ? sm.parked[w] : 0);
        any |= w < nwaves ? sm.has_list[w] : 0;
    }
    const int n = pre[kStreamWaves];
    const int nchunks = (n + kWave - 1) >> 6;
    u64 part = 0;
    bool have = false;
    for (int c = (wave - fin_wave) & (nwaves - 1); c < nchunks; c += nwaves) {
        const int i = c * kWave + lane;
        u64 key = 0;
        if (i < n) {
            int w = 0, first = 0;
#pragma unroll
            for (int j = 1; j < kStreamWaves; ++j)
                if (i >= pre[j]) {
                    w = j;
                    first = pre[j];
                }
            key = sm.stage[w][i - first];
        }
        const u64 sorted = sort64_desc<u64, true>(key);
        part = have ? merge_desc<u64, true>(part, sorted) : sorted;
        have = true;
    }
    if (nchunks <= 1 && !any) return part;            // the whole row was one chunk of fin_wave's
    if (mine_has) {
        part = have ? merge_desc<u64, true>(part, list) : list;
        have = true;
    }
    sm.wl[wave][lane] = part;
    __syncthreads();
    if (wave == fin_wave) {
        for (int w = 1; w < nwaves; ++w) {
            const u64 other = sm.wl[(wave + w) & (nwaves - 1)][lane];
            if (read_lane(other, 0) != 0) {
                part = have ? merge_desc<u64, true>(part, other) : other;
                have = true;
            }
        }
    }
    return part;
}

// ---------------------------------------------------------------------------
// constraint bookkeeping (Sec. 3.1): in-order phrases, one phrase under way
// ---------------------------------------------------------------------------
// Wave-wide, one lane per phrase: what the hypothesis (nmet tokens met, incomplete phrases inc,
// phrase ip under way with iq tokens met and next token nxt) may place now (Alg. 2 inner loop,
// Sec. 3.1 item 2) - the next token of the phrase under way, the first token of a phrase
// neither complete nor under way.  Of equal tokens only the lowest phrase keeps its entry
// (they are one coordinate).  Returns the lane's token or -1, and in bank the constraints met
// once it is placed: nmet+1 if it continues the phrase under way or no phrase is under way,
// else the phrase under way is unwound first (Sec. 3.1, last paragraph).
// ftok = first token of the lane's phrase, sfl = lower phrases with the same first token.
__device__ __forceinline__ int expandable_entry(int P, int nmet, u64 inc, int ip, int iq, int nxt, int ftok,
                                                u64 sfl, int &bank)
{
    const int lane = lane_id();
    const bool offers_first = lane < P && ((inc >> lane) & 1ull) && lane != ip;
    const u64 F = __ballot(offers_first);
    int w = -1;
    if (lane == ip) w = nxt;
    else if (offers_first && !(sfl & F)) w = ftok;
    if (ip >= 0) {
        const u64 E = __ballot(w >= 0 && lane != ip && w == nxt);   // at most one lane
        if (E) {
            const int lowest = __ffsll((long long)E) - 1;
            if (lowest < ip) {
                if (lane == ip) w = -1;
            } else if (lane == lowest) {
                w = -1;
            }
        }
    }
    bank = (ip < 0 || lane == ip || w == nxt) ? nmet + 1 : nmet - iq + 1;
    return w;
}

// ---------------------------------------------------------------------------
// allocation (Sec. 3.2) on one wavefront, registers only
// ---------------------------------------------------------------------------
// Lane x holds bank x (x < 64); bank 64 is carried wave-uniform.  c = candidates
// in the bank; returns the slots of the lane's bank and writes bank 64's to a64.
// Base split: floor(k/(C+1)) each, remainder to bank C.  Adjustment: banks with
// more slots than candidates, in ascending order, keep what they can fill and
// pass the rest to banks with spare candidates, nearest first, the higher
// neighbour before the lower, as much as each can take.
// adjust = false (Sec. 5): the base split stays; a bank keeps only the slots it can fill.
__device__ __forceinline__ int allocate_wave(int k, int C, int c, int c64, int &a64, bool adjust)
{
    const int lane = lane_id();
    const int base = k / (C + 1);
    const int rem = k - base * (C + 1);
    int a = (lane <= C) ? base + (lane == C ? rem : 0) : 0;
    a64 = (C == 64) ? base + rem : 0;
    if (lane > C) c = 0;
    if (C < 64) c64 = 0;
    if (!adjust) {
        a64 = min(a64, c64);
        return min(a, c);
    }

    u64 donors = __ballot(a > c);                         // fixed before the hand-outs begin:
    bool donor64 = a64 > c64;                             // a receiver never becomes a donor
    for (;;) {
        int b, e;
        if (donors != 0) {
            b = __ffsll((long long)donors) - 1;
            donors &= donors - 1;
            e = __builtin_amdgcn_readlane(a - c, b);
            if (lane == b) a = c;
        } else if (donor64) {
            donor64 = false;
            b = 64;
            e = a64 - c64;
            a64 = c64;
        } else {
            break;
        }
        const int need = max(0, c - a);
        const int need64 = max(0, c64 - a64);
        if (__ballot(need > 0) == 0 && need64 == 0) continue;   // nobody can take a slot
        // lane l looks at distance d = l+1: bank b+d first, then bank b-d
        const int d = lane + 1;
        const int xu = b + d, xd = b - d;
        const int nu = __shfl(need, xu & 63, kWave);
        const int nd = __shfl(need, xd & 63, kWave);
        const int up = (xu <= C) ? (xu < 64 ? nu : need64) : 0;
        const int dn = (xd >= 0) ? nd : 0;
        const int before = wave_inclusive_sum(up + dn) - (up + dn);
        const int gu = min(up, max(0, e - before));
        const int gd = min(dn, max(0, e - before - up));
        const int from_up = __shfl(gu, (lane - b - 1) & 63, kWave);
        const int from_dn = __shfl(gd, (b - lane - 1) & 63, kWave);
        if (lane > b) a += from_up;
        if (lane < b) a += from_dn;
        if (b < 64) a64 += __builtin_amdgcn_readlane(gu, 63 - b);   // 0 unless C == 64
    }
    return a;
}

// ---------------------------------------------------------------------------
// merge phase
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 pack_sel(int met_bits, int bank, uint32_t ord, uint32_t flat)
{
    const int fb = 32 - met_bits;
    const uint32_t flatmask = fb >= 32 ? 0xFFFFFFFFu : ((1u << fb) - 1u);
    u64 v = ((u64)ord << fb) | (u64)(flatmask - flat);
    if (met_bits) v |= (u64)bank << (64 - met_bits);
    return v;
}

// stream-phase key (score image << 32 | ~flat) -> selection key in bank `bank` (its body - score image
// << fb | ~flat in fb bits - orders like the stream-phase key); 0 stays 0
__device__ __forceinline__ u64 sel_from_rowkey(int met_bits, int bank, u64 key)
{
    if (key == 0) return 0;
    return pack_sel(met_bits, bank, (uint32_t)(key >> 32), key_flat(key));
}

// The phrases whose first token is w (w < 0: none), as a bit mask.  Every lane looks its own
// token up in the bucket of the token's low six bits: one trip to LDS where the bucket's
// phrases all begin with the same token (nearly always), else they are compared one by one.
__device__ __forceinline__ u64 first_token_matches(int w, const MergeSmem &sm)
{
    if (w < 0) return 0;
    const int same = sm.btok[w & 63];
    u64 todo = sm.fbucket[w & 63];
    if (same == w) return todo;
    u64 mine = 0;
    if (same == -2) {
        while (todo) {
            const int j = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            if (sm.ct.tok[sm.ct.poff[j]] == w) mine |= 1ull << j;
        }
    }
    return mine;
}

// Constraints met after a hypothesis (nmet met, phrase ip under way with iq tokens) emits a
// token: is_next = it continues the phrase under way; match = phrases it could begin;
// inc = phrases not complete.
__device__ __forceinline__ int nmet_after(int nmet, int ip, int iq, bool is_next, u64 match, u64 inc)
{
    if (ip >= 0 && is_next) return nmet + 1;
    const int base = ip >= 0 ? nmet - iq : nmet;          // a broken phrase is unwound
    return base + ((match & inc) ? 1 : 0);
}

// The 64 greatest 32-bit keys of the rows of one wave (row i of the wave = list(i), a
// decreasing list; rows are dealt out to the waves in turn, those from k on are empty).  Two
// chains of merges run side by side, so that their instructions interleave, and are joined at
// the end.  A list whose head is below place `kth` of the chain it would join cannot change
// places 0..kth of the result and may be skipped (LOOK); apart from that the result is exact.
template <int R, int MW, bool LOOK, typename List>
__device__ __forceinline__ uint32_t wave_best64(int wave, int k, int kth, List list, uint32_t &fell)
{
    uint32_t a0 = wave < k ? list(0) : 0u;
    uint32_t a1 = (R > 1 && wave + MW < k) ? list(R > 1 ? 1 : 0) : 0u;
#pragma unroll
    for (int i = 2; i < R; i += 2) {
        if (wave + i * MW < k) {               // wave-uniform
            const bool pair = i + 1 < R && wave + (i + 1) * MW < k;
            const uint32_t s0 = list(i);
            const uint32_t s1 = pair ? list(i + 1 < R ? i + 1 : i) : 0u;
            // LOOK: lists are looked at before they are merged (worth it where many are empty or
            // weak, or a wave has many rows); otherwise every row that exists is merged, and no
            // value decides a branch
            bool n0 = true, n1 = pair;
            if (LOOK) {
                const uint32_t h0 = (uint32_t)__builtin_amdgcn_readlane((int)s0, 0);
                const uint32_t h1 = (uint32_t)__builtin_amdgcn_readlane((int)s1, 0);
                n0 = h0 != 0 && h0 >= (uint32_t)__builtin_amdgcn_readlane((int)a0, kth);
                n1 = h1 != 0 && h1 >= (uint32_t)__builtin_amdgcn_readlane((int)a1, kth);
            }
            if (n0 && n1) {
                a0 = merge32_desc(a0, s0, fell);
                a1 = merge32_desc(a1, s1, fell);
            } else if (n0) {
                a0 = merge32_desc(a0, s0, fell);
            } else if (n1) {
                a1 = merge32_desc(a1, s1, fell);
            }
        }
    }
    if (LOOK) return __builtin_amdgcn_readlane((int)a1, 0) != 0 ? merge32_desc(a0, a1, fell) : a0;
    return (R > 1 && wave + MW < k) ? merge32_desc(a0, a1, fell) : a0;
}

// The 64 greatest keys of the lists the MW waves have left in buf (after a barrier), for the
// calling wave: a tree of merges whose independent pairs run side by side.
template <int MW>
__device__ __forceinline__ uint32_t join_best64(const uint32_t (&buf)[kMergeWavesMax][kWave], int wave, int lane,
                                                uint32_t &fell)
{
    uint32_t o[MW];
#pragma unroll
    for (int w = 0; w < MW; ++w) o[w] = buf[(wave + w) & (MW - 1)][lane];
#pragma unroll
    for (int span = 1; span < MW; span *= 2)
#pragma unroll
        for (int w = 0; w + span < MW; w += 2 * span) o[w] = merge32_desc(o[w], o[w + span], fell);
    return o[0];
}

// The same where most lists are expected to be empty (an empty list costs nothing), in every
// wave; one barrier.
template <int MW>
__device__ __forceinline__ uint32_t block_best64_sparse(uint32_t (&buf)[kMergeWavesMax][kWave], int wave, int lane,
                                                        uint32_t mine, uint32_t &fell)
{
    buf[wave][lane] = mine;
    __syncthreads();
    uint32_t acc = mine;
#pragma unroll
    for (int w = 1; w < MW; ++w) {
        const uint32_t other = buf[(wave + w) & (MW - 1)][lane];
        if (__builtin_amdgcn_readlane((int)other, 0) != 0) acc = merge32_desc(acc, other, fell);
    }
    return acc;
}

// MW: waves of the sentence's workgroup; ROWS: beam rows per wave the code is laid out for
// (k <= MW * ROWS; wave w takes rows w, w + MW, ...): the loops over a wave's rows are unrolled, so a
// smaller bound keeps the code of small beams short.
// rowlists, conskeys, k: what the first loads need (p.rowlists, p.conskeys and p.k, handed over apart).
template <int ROWS, int MW>
__device__ __forceinline__ void merge_phase(const StepParams &p, const u64 *rowlists, const u64 *conskeys, int k,
                                            int b, MergeSmem &sm, u64 *cand)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // in a scalar register: row guards are scalar branches
    // the row lists first: the chain of this phase starts with them, and their addresses need nothing
    // that has to be read from memory first
    constexpr int kRowsPerWave = ROWS;
    u64 rl[kRowsPerWave], ck[kRowsPerWave];
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) {
        const int h = wave + i * MW;
        rl[i] = 0;
        if (h < k) {
            const size_t o = ((size_t)b * k + h) * kWave + lane;
            rl[i] = rowlists[o];
        }
    }
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) {
        const int h = wave + i * MW;
        ck[i] = 0;
        if (h < k) {
            const size_t o = ((size_t)b * k + h) * kWave + lane;
            ck[i] = conskeys[o];
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    const int mb = p.met_bits;
    const int sel_shift = 64 - mb;
    const u64 body_mask = mb ? ((1ull << sel_shift) - 1ull) : ~0ull;
    const int fb = 32 - mb;
    const uint32_t flatmask = fb >= 32 ? 0xFFFFFFFFu : ((1u << fb) - 1u);
    const uint32_t tokmask = (1u << p.tok_bits) - 1u;

    // ---- everything this sentence needs from memory, requested at once: every load is issued
    // before the first one is waited for (clamped indices instead of branches) --------------
    const int t64 = tid < kMaxCons ? tid : kMaxCons;
    const int hs = tid < k ? tid : k - 1;
    const size_t rs = (size_t)b * k + hs;
    const int ld_poff = p.phr_off[(size_t)b * (kMaxCons + 1) + t64];
    const int ld_tok = p.cons_tok[(size_t)b * kMaxCons + lane];
    const int P = p.nphr[b];
    const u64 ld_bucket = p.first_bucket[(size_t)b * kMaxCons + lane];
    const int ld_btok = p.bucket_tok[(size_t)b * kMaxCons + lane];
    const u64 ld_met = p.met_cur[rs];
    const u64 ld_inc = p.inc_cur[rs];
    const int ld_ipq = p.ipq_cur[rs];
    const int ld_nxt = p.nxt_cur[rs];
    const int ld_len = p.len_cur[rs];
    const int ld_fin = p.fin_cur[rs];
    // every load above is on its way before anything waits for one of them: the lists are
    // pinned here, or their loads would be moved down to the conditional code that uses them
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) asm volatile("" : "+v"(rl[i]), "+v"(ck[i]));
    // ---- source 1: the sentence's k best (Sec. 3.1 item 1) = top k of the union of the row
    // lists.  All that is needed of them is the bar tau a key has to reach to be among them.
    // The k-th best SCORE comes from merging the 32-bit score images alone.  If the keys with
    // that score or a better one are exactly k, that is the bar.  Otherwise several keys tie
    // for the last places: the same merge over the low words (the coordinates, complemented)
    // of the keys with that score finds the last one that gets in. -------------------------
    uint32_t fell = 0;
    uint32_t accs = wave_best64<kRowsPerWave, MW, (kRowsPerWave > 4)>(wave, k, k - 1, [&](int i) { return (uint32_t)(rl[i] >> fb); }, fell);
    // the sentence's tables and beam go to LDS only now: their loads were issued after those of the
    // row lists and arrive later, and the merges above needed none of them
    if (tid <= kMaxCons) sm.ct.poff[tid] = ld_poff;
    if (tid < 2 * kMaxCons) {
        sm.cnt[tid] = 0;
        sm.alloc[tid] = 0;                             // banks beyond the sentence's get no slot
        sm.start[tid] = 0;
    }
    if (tid < kMaxCons) {
        sm.ct.tok[tid] = ld_tok;
        sm.fbucket[tid] = ld_bucket;
        sm.btok[tid] = ld_btok;
        sm.sel[tid] = 0;                               // places beyond the last selected key compare as empty
    }
    if (tid == 0) {
        sm.ncand = 0;
        sm.nsel = 0;
        sm.kept = 0;
    }
    if (tid < k) {
        HypState hs;
        hs.met = ld_met;
        hs.inc = ld_inc;
        hs.ipq = ld_ipq;
        hs.nxt = ld_nxt;
        hs.len = ld_len;
        hs.misc = (ld_fin & kFinFinished) | (__popcll(ld_met) << 8);
        sm.hyp[tid] = hs;
    }
    sm.wf[wave][lane] = fell;
    sm.ws[wave][lane] = accs;
    __syncthreads();                                       // tables and beam are in LDS too
    const int C = sm.ct.poff[P];
    // The sentence's best score images, lane i = i-th best, from the waves' lists.  With eight
    // waves two share a SIMD, and the join is the same work in every wave: the first four (one
    // per SIMD) do it and hand the outcome to the others.
    constexpr int kJoiners = MW < 4 ? MW : 4;
    uint32_t tau_s = 0;
    bool settled = true;
    int need = 0;                                          // places left for keys that tie at the bar's score
    if (wave < kJoiners) {
        accs = join_best64<MW>(sm.ws, wave, lane, fell);
        tau_s = (uint32_t)__builtin_amdgcn_readlane((int)accs, k - 1);
        if (tau_s != 0) {
            settled = (int)__popcll(__ballot(accs >= tau_s)) == k;  // places k.. hold lower scores
            if (settled && k == kWave) {
                // every place is taken: a tie may hide among the keys the merges dropped
                for (int w = 1; w < MW; ++w) {
                    const uint32_t f = sm.wf[(wave + w) & (MW - 1)][lane];
                    fell = fell > f ? fell : f;
                }
                settled = wave_max_u32(fell) < tau_s;
            }
        }
        need = k - __popcll(__ballot(accs > tau_s));
        if (MW > kJoiners && tid == 0) {
            sm.bar_score = tau_s;
            sm.bar_need = settled ? -1 : need;
        }
    }
    if (MW > kJoiners) {
        __syncthreads();
        tau_s = sm.bar_score;
        need = sm.bar_need;
        settled = need < 0;
    }
    // tau = what a selection-key body has to reach to be among the k best; 0 while fewer than
    // k finite sums exist, in which case every finite sum is among them.
    u64 tau = (u64)tau_s << fb;
    if (!settled) {                                        // the same decision in every wave
        const uint32_t low_bias = fb < 32 ? 1u : 0u;
        uint32_t unused = 0;
        uint32_t accl = wave_best64<kRowsPerWave, MW, true>(wave, k, need - 1, [&](int i) {
            // the tied keys of a decreasing list are neighbours: move them to the front
            // (a low word may be 0 where it has fewer than 32 bits: one is added meanwhile)
            const uint32_t hi = (uint32_t)(rl[i] >> fb);
            if (__ballot(hi == tau_s) == 0) return 0u;     // most rows hold none
            const int first = __popcll(__ballot(hi > tau_s));
            const uint32_t lo = hi == tau_s ? ((uint32_t)rl[i] & flatmask) + low_bias : 0u;
            const uint32_t moved = (uint32_t)__shfl((int)lo, (lane + first) & (kWave - 1), kWave);
            return lane + first < kWave ? moved : 0u;
        }, unused);
        accl = block_best64_sparse<MW>(sm.ws2, wave, lane, accl, unused);
        const uint32_t tau_l = (uint32_t)__builtin_amdgcn_readlane((int)accl, need - 1);
        tau = ((u64)tau_s << fb) | (u64)(tau_l - low_bias);
    }

    // ---- candidates, deduplicated by construction: the k best; a row's best (item 3, the
    // head of its list) unless among the k best; an expandable constraint token (item 2)
    // unless among the k best or equal to its row's best (the table never offers one token
    // twice for a hypothesis).  Each wave collects what its own rows give to sources 1 and 3
    // (in a decreasing list the keys that reach tau come first), works out their banks with
    // add() (Sec. 3.1), counts its candidates, reserves room with one atomic and writes them.
    // Lanes count what they hold themselves; two prefix sums over the wave then give every lane
    // its places (no wave-wide vote per row).
    const bool by_score = settled && tau_s != 0;
    // a key of a row's list is kept if it reaches tau; lane 0 holds the row's best and keeps any
    const u64 keep_from = lane == 0 ? 1ull : (tau > 1 ? tau : 1ull);
    // a constraint token is a candidate while below tau.  Where tau stands for a score alone,
    // one with exactly that score is among the k best only if its row's list holds it (every
    // listed key with that score is): those pass for now and are looked up below.
    const u64 below = by_score ? tau + (1ull << fb) : tau;
    uint32_t gm = 0, cm = 0;                               // bit i: this lane's key of row i is kept
    bool some_tied = false;
    if (tau != 0) {
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            if (wave + i * MW < k) {
                const u64 best = read_lane(rl[i], 0) & body_mask;
                gm |= ((rl[i] & body_mask) >= keep_from ? 1u : 0u) << i;
                const u64 body = ck[i] & body_mask;
                const bool valid = body - 1 < below - 1 && body != best;      // (an empty place holds 0)
                cm |= (valid ? 1u : 0u) << i;
                if (by_score) some_tied |= valid && body >= tau;
            }
        }
    } else {
        // fewer than k finite sums: all of them are among the k best, none is left for source 2
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i)
            if (wave + i * MW < k) gm |= (rl[i] != 0 ? 1u : 0u) << i;
    }
    if (__ballot(some_tied)) {                             // rare
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            if (wave + i * MW < k) {
                const u64 body = ck[i] & body_mask;
                u64 tied = __ballot(((cm >> i) & 1u) != 0 && body >= tau);
                while (tied) {
                    const int l = __ffsll((long long)tied) - 1;
                    tied &= tied - 1;
                    const u64 one = read_lane(body, l);
                    if (__ballot((rl[i] & body_mask) == one) != 0 && lane == l) cm &= ~(1u << i);
                }
            }
        }
    }
    // Both kinds of key arrive with their bank (the constraints met once the token is placed, worked
    // out with add() by the row's own workgroup, Sec. 3.1), so a kept key goes straight to its place.
    const int g = __popc(gm), c = __popc(cm);              // this lane's keys from sources 1 and 3, from source 2
    const int g_incl = wave_inclusive_sum(g), c_incl = wave_inclusive_sum(c);
    const int n13_all = __builtin_amdgcn_readlane(g_incl, kWave - 1);
    const int total = n13_all + __builtin_amdgcn_readlane(c_incl, kWave - 1);
    int at = 0;
    if (lane == 0 && total > 0) at = atomicAdd(&sm.ncand, total);
    at = __builtin_amdgcn_readfirstlane(at);
    // The count cannot exceed the room (at most k keys reach tau, a row adds one more only if none of
    // its keys does, the host sized `cand` for every source) as long as the row lists are what the
    // stream phase writes: decreasing, distinct keys.  A wave that finds otherwise writes nothing: a
    // damaged list costs a wrong beam, not a stray write.  (The bank tables hold every value the
    // bank field of a key can take.)
    if (at + total <= p.cand_cap) {
        int to = at + g_incl - g;
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            if (wave + i * MW < k && ((gm >> i) & 1u)) {
                cand[to++] = rl[i];
                atomicAdd(&sm.cnt[mb ? (int)(rl[i] >> sel_shift) : 0], 1);    // bank = constraints met (Sec. 3.1)
            }
        }
        to = at + n13_all + c_incl - c;
#pragma unroll
        for (int i = 0; i < kRowsPerWave; ++i) {
            if (wave + i * MW < k && ((cm >> i) & 1u)) {
                cand[to++] = ck[i];
                atomicAdd(&sm.cnt[mb ? (int)(ck[i] >> sel_shift) : 0], 1);
            }
        }
    }
    __syncthreads();
    const int ncand = min(sm.ncand, p.cand_cap);
    const int nchunks = (ncand + kWave - 1) >> 6;

    // ---- slots per bank (Sec. 3.2) --------------------------------------------------------
    if (wave == 0) {
        const int c = sm.cnt[lane];
        const int c64 = sm.cnt[kMaxCons];
        int a64;
        const int a = allocate_wave(k, C, c, c64, a64, p.adjust != 0);
        sm.alloc[lane] = a;
        if (lane == 0) sm.alloc[kMaxCons] = a64;
        const int cc = lane <= C ? c : 0;
        const int incl = wave_inclusive_sum(cc);          // candidates in banks <= lane
        const int total63 = __builtin_amdgcn_readlane(incl, 63);
        const int c64v = C == 64 ? c64 : 0;
        sm.start[lane] = (total63 - incl) + c64v;         // candidates in higher banks
        if (lane == 0) sm.start[kMaxCons] = 0;
    }
    // ---- every candidate's place in the order (bank desc, score desc, coordinate asc):
    // chunks of 64 are sorted by one wave each (wave 0, busy with the allocation, last); a
    // candidate's rank is its place in its own chunk plus, by a search with three probes a round,
    // the keys greater than it in every other chunk ------------------------------------------------------------
    const int my_first = MW - 1 - wave;
    for (int c = my_first; c < nchunks; c += MW) {
        const int i = c * kWave + lane;
        cand[i] = sort64_desc<u64, true>(i < ncand ? cand[i] : 0ull);
    }
    __syncthreads();
    for (int c = my_first; c < nchunks; c += MW) {
        const u64 mine = cand[c * kWave + lane];
        int rank = lane;
        // four searches at a time, so that their LDS reads overlap
        for (int c0 = 0; c0 < nchunks; c0 += 4) {
            int pos[4];
            bool full[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c2 = c0 + q < nchunks ? c0 + q : c;     // out of range: own chunk, ignored below
                pos[q] = 0;
                full[q] = cand[c2 * kWave + 63] > mine;
            }
            // three probes a round (quarters, then sixteenths, then single places): three
            // dependent trips to LDS instead of six
#pragma unroll
            for (int step = 16; step >= 1; step >>= 2) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c2 = c0 + q < nchunks ? c0 + q : c;
                    const u64 *at0 = cand + c2 * kWave + pos[q] - 1;
                    const int above = (at0[step] > mine ? 1 : 0) + (at0[2 * step] > mine ? 1 : 0) +
                                      (at0[3 * step] > mine ? 1 : 0);
                    pos[q] += step * above;
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (c0 + q < nchunks && c0 + q != c) rank += full[q] ? 64 : pos[q];
        }
        if (mine != 0) {
            const int bank = mb ? (int)(mine >> sel_shift) : 0;
            // within a bank the best alloc[bank] are taken (Sec. 3.1/3.2)
            if (rank - sm.start[bank] < sm.alloc[bank]) {
                const int place = atomicAdd(&sm.nsel, 1);
                if (place < kMaxBeam) sm.sel[place] = mine & body_mask;
            }
        }
    }
    __syncthreads();

    // ---- new beam, best first (Sec. 3.1); empty slots last ---------------------------------
    // One lane per selected candidate.  Its place in the new beam is the number of selected keys greater
    // than its own (at most 64 uniform LDS reads: cheaper than a 64-lane sort); wave 1 counts that
    // while wave 0 takes the hypotheses through add().
    const int nsel = min(sm.nsel, k);
    const bool live = lane < nsel;
    const u64 mine = (wave <= 1 && live) ? sm.sel[lane] : 0ull;
    if (wave == 1) {
        int slot = 0;
        for (int j = 0; j < nsel; j += 4)                 // (kMaxBeam is a multiple of 4; unused places hold 0)
            slot += (sm.sel[j] > mine ? 1 : 0) + (sm.sel[j + 1] > mine ? 1 : 0) + (sm.sel[j + 2] > mine ? 1 : 0) +
                    (sm.sel[j + 3] > mine ? 1 : 0);
        sm.slot[lane] = slot;
    }
    int token = p.pad_id, parent = -1, length = 0, ipq2 = -1, nxt2 = -1;
    float score = -INFINITY;
    u64 met2 = 0, inc2 = 0;
    uint8_t flags = 2, fin2 = 0;
    if (wave == 0) {
        if (live) {
            const uint32_t code = flatmask - ((uint32_t)mine & flatmask);
            parent = (int)(code >> p.tok_bits);
            token = (int)(code & tokmask);
            score = float_from_ord((uint32_t)(mine >> fb));
        }
        const u64 match = first_token_matches(live ? token : -1, sm);
        if (live) {
            const HypState hs = sm.hyp[min(parent, kMaxBeam - 1)];
            met2 = hs.met;
            inc2 = hs.inc;
            const int ipq = hs.ipq;
            int ip = ipq < 0 ? -1 : (ipq >> 8), iq = ipq < 0 ? 0 : (ipq & 255);
            const bool pfin = (hs.misc & kFinFinished) != 0;
            if (!pfin) {
                // add(token), Sec. 3.1: advance the phrase under way, or unwind it and let the
                // token begin the lowest-index incomplete phrase that starts with it
                if (ip >= 0 && token == hs.nxt) {
                    const int o = sm.ct.poff[ip];
                    met2 |= 1ull << (o + iq);
                    ++iq;
                    if (o + iq == sm.ct.poff[ip + 1]) {
                        inc2 &= ~(1ull << ip);
                        ip = -1;
                        iq = 0;
                    }
                } else {
                    if (ip >= 0) {
                        met2 &= ~(((1ull << iq) - 1ull) << sm.ct.poff[ip]);
                        ip = -1;
                        iq = 0;
                    }
                    const u64 startable = match & hs.inc;
                    if (startable) {
                        const int j = __ffsll((long long)startable) - 1;
                        const int o = sm.ct.poff[j];
                        met2 |= 1ull << o;
                        if (sm.ct.poff[j + 1] - o > 1) {
                            ip = j;
                            iq = 1;
                        } else {
                            inc2 &= ~(1ull << j);
                        }
                    }
                }
            }
            ipq2 = ip < 0 ? -1 : ((ip << 8) | iq);
            nxt2 = ip < 0 ? -1 : sm.ct.tok[sm.ct.poff[ip] + iq];
            fin2 = (pfin || token == p.eos_id) ? 1 : 0;
            length = pfin ? hs.len : hs.len + 1;
            flags = fin2;
            // Sec. 4: a hypothesis that completes now is kept with its score per word (one fp32
            // division, the length counts end-of-sentence); it competed with its raw sum above
            if (p.normalize && fin2 && !pfin) score = __fdiv_rn(score, (float)length);
        }
    }
    __syncthreads();
    if (wave == 0) {
        int slot = sm.slot[lane];
        // Sec. 4 / Sec. 6.3: hypotheses, completed or not, below (best completed - threshold) leave
        // the beam; the others close ranks
        bool keep = live;
        int nlive = nsel;
        if (p.prune >= 0.0f) {
            float best = (live && fin2) ? score : -INFINITY;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) best = fmaxf(best, __shfl_xor(best, d, kWave));
            if (best > -INFINITY) keep = live && score >= best - p.prune;
            if (keep) atomicOr(&sm.kept, 1ull << slot);
            // every lane's OR belongs to the one LDS instruction issued before this read
            const u64 km = __hip_atomic_load(&sm.kept, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            slot = __popcll(km & ((1ull << slot) - 1ull));
            nlive = __popcll(km);
        }
        const u64 open = __ballot(keep && !fin2);
        if (keep) {
            const size_t o = (size_t)b * k + slot;
            p.score_nxt[o] = score;
            p.met_nxt[o] = met2;
            p.inc_nxt[o] = inc2;
            p.ipq_nxt[o] = ipq2;
            p.nxt_nxt[o] = nxt2;
            p.len_nxt[o] = length;
            p.fin_nxt[o] = (uint8_t)(fin2 | ((!fin2 && (int)__popcll(met2) < C) ? kFinEosBlocked : 0));
            p.hist_token[o] = token;
            p.hist_backptr[o] = parent;
            if (p.out_token) p.out_token[o] = token;
            if (p.out_backptr) p.out_backptr[o] = parent;
            if (p.out_score) p.out_score[o] = score;
            if (p.out_flags) p.out_flags[o] = flags;
        }
        if (lane >= nlive && lane < k) {                  // empty slots
            const size_t o = (size_t)b * k + lane;
            p.score_nxt[o] = -INFINITY;
            p.met_nxt[o] = 0;
            p.inc_nxt[o] = 0;
            p.ipq_nxt[o] = -1;
            p.nxt_nxt[o] = -1;
            p.len_nxt[o] = 0;
            p.fin_nxt[o] = 0;
            p.hist_token[o] = p.pad_id;
            p.hist_backptr[o] = -1;
            if (p.out_token) p.out_token[o] = p.pad_id;
            if (p.out_backptr) p.out_backptr[o] = -1;
            if (p.out_score) p.out_score[o] = -INFINITY;
            if (p.out_flags) p.out_flags[o] = 2;
        }
        const u64 closed = __ballot(keep && fin2);
        if (p.track && closed != 0) {
            // Sec. 3.3: a completed hypothesis may lose its slot later on, so the best one seen so
            // far is remembered: value per word (the stored score where the beam already holds it
            // per word), replaced only by a strictly better one - the earliest step, then the
            // lowest slot keep a tie.  A hypothesis carried along compares equal to its own record.
            const bool cl = keep && fin2;
            const float q = !cl ? -INFINITY : (p.normalize ? score : __fdiv_rn(score, (float)length));
            float best = q;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) best = fmaxf(best, __shfl_xor(best, d, kWave));
            int first = (cl && q == best) ? slot : kWave;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) first = min(first, __shfl_xor(first, d, kWave));
            if (cl && slot == first) {
                BestCompleted *r = p.best + b;
                if (!r->have || best > r->q) {
                    r->have = 1;
                    r->step = p.step;
                    r->slot = slot;
                    r->len = length;
                    r->q = best;
                    r->score = score;
                }
            }
        }
        if (lane == 0)                                    // stopping tests: Sec. 4 (all), Sec. 6.3 (any)
            p.all_finished[b] = (uint8_t)(((nlive > 0 && open == 0) ? 1 : 0) | (closed != 0 ? 2 : 0));
    }
}

}  // namespace dba
