// Device side of the DBA step (Post & Vilar 2018, Alg. 2, Sec. 3.1-3.3) for gfx950.
//
// Two phases per step:
//   stream phase  one workgroup per beam row (b,h): a single pass over the V
//                 log-probs of that row - score add, end-of-sentence mask,
//                 exact top-64 of the row (which holds the row's best token
//                 and its share of the sentence's top-k) - written as one
//                 sorted 64-key list per row;
//   merge phase   one workgroup per sentence: sentence top-k from the row
//                 lists, constraint-token gather, state transition add(),
//                 dedup, banks, allocation with adjustment, selection, new
//                 beam.  In the fused launch it is run by whichever row
//                 workgroup of the sentence finishes last.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "wave_topk.hpp"

namespace dba {

constexpr int kMaxBeam = 64;
constexpr int kMaxCons = 64;          // constraint tokens (and phrases) per sentence
constexpr int kBlock = 256;           // threads per workgroup
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kSortThresh = 10;       // survivors in one wave-wide test above which a sort+merge beats serial inserts

struct StepParams {
    int B, k, V;
    int eos_id, pad_id;
    int met_bits;                     // width of the bank field in the packed selection key
    int fused;                        // 1: the last row workgroup of a sentence runs the merge phase
    const float *logp;                // [B,k,V]
    // beam before the step
    const float *score_cur;           // [B,k]  (-inf: empty slot)
    const u64 *met_cur;               // [B,k]  bit i = constraint token i met
    const int32_t *ipq_cur;           // [B,k]  phrase under way * 256 + tokens met in it, or -1
    const int32_t *len_cur;           // [B,k]
    const uint8_t *fin_cur;           // [B,k]
    // beam after the step
    float *score_nxt;
    u64 *met_nxt;
    int32_t *ipq_nxt;
    int32_t *len_nxt;
    uint8_t *fin_nxt;
    // constraints
    const int32_t *cons_tok;          // [B,64]
    const int32_t *phr_off;           // [B,65] token offset of each phrase, phr_off[b][P] = C
    const int32_t *nphr;              // [B]
    // scratch
    u64 *rowlists;                    // [B*k,64]
    unsigned int *counters;           // [B] rows of the sentence that have delivered their list
    // outputs (each may be null)
    int32_t *out_token, *out_backptr;
    float *out_score;
    uint8_t *out_flags;
    int32_t *hist_token, *hist_backptr;   // row t of the history, [B,k]
};

struct MergeSmem {
    u64 wl[kWavesPerBlock][kWave];
    u64 t1[kWave];
    u64 rb[kMaxBeam];
    u64 sel[kMaxBeam];
    u64 met[kMaxBeam];
    float prev[kMaxBeam];
    int ipq[kMaxBeam];
    int len[kMaxBeam];
    int tok[kMaxCons];
    int poff[kMaxCons + 1];
    int cnt[kMaxCons + 1];
    int alloc[kMaxCons + 1];
    int start[kMaxCons + 1];
    unsigned char fin[kMaxBeam];
    int nsel;
    int last;
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

__device__ __forceinline__ v4f neg_inf4()
{
    return v4f{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
}

// max of four finite-or-infinite floats in two instructions (the inputs are never NaN, so the
// quieting moves a generic fmaxf would add are not needed)
__device__ __forceinline__ float max4(const v4f &x)
{
    float t, m;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(t) : "v"(x.x), "v"(x.y), "v"(x.z));
    asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(t), "v"(x.w));
    return m;
}

// The log-probs are read exactly once: non-temporal loads keep them from displacing
// anything useful in the caches.
template <int U>
__device__ __forceinline__ void load_tile(const v4f *__restrict__ vec, int nv, int tile, int lane,
                                          v4f (&x)[U])
{
    const int base = tile * (kWave * U);
    if (base + kWave * U <= nv) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = __builtin_nontemporal_load(vec + base + u * kWave + lane);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = base + u * kWave + lane;
            x[u] = (i < nv) ? __builtin_nontemporal_load(vec + i) : neg_inf4();
        }
    }
}

// Sec. 3.3: while constraints are unmet the end-of-sentence entry does not exist.  rel = its
// position inside the tile in floats (wave-uniform); the one lane holding it drops it.
template <int U>
__device__ __forceinline__ void block_eos(v4f (&x)[U], int rel, int lane)
{
    const int uu = rel / (4 * kWave), ln = (rel >> 2) & (kWave - 1), c = rel & 3;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u == uu && lane == ln) {
            if (c == 0) x[u].x = -INFINITY;
            if (c == 1) x[u].y = -INFINITY;
            if (c == 2) x[u].z = -INFINITY;
            if (c == 3) x[u].w = -INFINITY;
        }
    }
}

// LDS shared by the waves of one row's workgroup during the stream phase.
struct StreamSmem {
    u64 wl[kWavesPerBlock][kWave];      // the waves' lists, for the final merge
    u64 stage[kWavesPerBlock][kStageCap];   // candidates parked between flushes
    uint32_t boot[kWavesPerBlock][kWave];   // sorted per-lane maxima of every wave's first tile (order images)
    unsigned int thr;                   // best bound any wave has published (order-preserving u32)
};

// One wave's share of one row: tiles wave, wave+nwaves, ... of 64*U float4 each.  Must be
// called by every thread of the workgroup (it contains one barrier).
//
// s = prev + logp is a single fp32 add.  An element is looked at closely only if its sum can
// still reach the row's k best (>=: a later element may tie the k-th score and win on the
// coordinate).  Rounding is monotone, so max(prev + x_i) == prev + max(x_i): one add per
// float4 decides whether any of its four elements needs a look.
//
// Thresholds.  (1) Every lane takes the maximum of its share of the wave's first tile; the
// k-th greatest of all the workgroup's per-lane maxima is a floor: k different lanes hold an
// element at least that large, so nothing below it can be among the row's k best.  (2) A wave
// whose own list holds k entries uses the score of its k-th, publishes it into sm.thr (atomic
// max on an order-preserving u32) and re-reads the workgroup's maximum once per tile.  Any
// wave's bound holds for the whole row, so a stale value only lets a few more elements
// through; it never drops one.  The row's best element is never below any bound, so it
// always survives.
template <int U>
__device__ __forceinline__ void stream_row(const float *__restrict__ row, int V, float prev,
                                           int eos_block, uint32_t flat_base, int kk, int wave,
                                           int nwaves, StreamSmem &sm, RowTop &st)
{
    const int lane = lane_id();
    const uintptr_t addr = reinterpret_cast<uintptr_t>(row);
    int head = (int)(((16u - (unsigned)(addr & 15u)) & 15u) >> 2);
    if (head > V) head = V;
    const int nv = (V - head) >> 2;
    const int tail = V - head - (nv << 2);
    const v4f *__restrict__ vec = reinterpret_cast<const v4f *>(row + head);
    const int ntiles = (nv + kWave * U - 1) / (kWave * U);
    const int eos_rel0 = eos_block >= 0 ? eos_block - head : -1;   // position in the aligned body

    v4f cur[U], nxt[U];
#pragma unroll
    for (int u = 0; u < U; ++u) nxt[u] = neg_inf4();
    int tl = wave;
    uint32_t boot = ord_from_float(-INFINITY);
    if (tl < ntiles) {
        load_tile<U>(vec, nv, tl, lane, cur);
        if (nwaves + tl < ntiles) load_tile<U>(vec, nv, tl + nwaves, lane, nxt);
        const int rel = eos_rel0 - tl * (4 * kWave * U);
        if (eos_rel0 >= 0 && rel >= 0 && rel < 4 * kWave * U) block_eos<U>(cur, rel, lane);
        float lane_max = max4(cur[0]);
#pragma unroll
        for (int u = 1; u < U; ++u) {
            const float mu = max4(cur[u]);
            asm("v_max_f32 %0, %1, %2" : "=v"(lane_max) : "v"(lane_max), "v"(mu));
        }
        boot = sort64_desc<uint32_t>(ord_from_float(prev + lane_max));
    }
    if (nwaves > 1) {
        sm.boot[wave][lane] = boot;
        __syncthreads();
        for (int w = 0; w < nwaves; ++w)
            if (w != wave) boot = merge_desc<uint32_t>(boot, sm.boot[w][lane]);
    }
    st.floor = float_from_ord((uint32_t)__builtin_amdgcn_readlane((int)boot, kk - 1));
    st.thr = fmaxf(st.floor, kLowestFinite);
    u64 *stage = sm.stage[wave];
    int cnt = 0;
    // one tile: test its U float4 groups, park what may belong to the top k
    auto examine = [&](const v4f (&t)[U], int tile) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const v4f x = t[u];
            if (__any(prev + max4(x) >= st.thr)) {
                const uint32_t flat0 = flat_base + (uint32_t)(head + 4 * ((tile * U + u) * kWave));
                const float s0 = prev + x.x, s1 = prev + x.y, s2 = prev + x.z, s3 = prev + x.w;
                const u64 m0 = __ballot(s0 >= st.thr);
                if (m0) stage_candidates(st, stage, cnt, s0, m0, flat0, 4u, kk);
                const u64 m1 = __ballot(s1 >= st.thr);
                if (m1) stage_candidates(st, stage, cnt, s1, m1, flat0 + 1u, 4u, kk);
                const u64 m2 = __ballot(s2 >= st.thr);
                if (m2) stage_candidates(st, stage, cnt, s2, m2, flat0 + 2u, 4u, kk);
                const u64 m3 = __ballot(s3 >= st.thr);
                if (m3) stage_candidates(st, stage, cnt, s3, m3, flat0 + 3u, 4u, kk);
            }
        }
    };
    // after a tile: start the load that refills its registers (two tiles ahead) and make the
    // other buffer ready (end-of-sentence mask, freshest shared bound)
    auto advance = [&](v4f (&done)[U], v4f (&next)[U], int next_tile) {
        if (next_tile + nwaves < ntiles) load_tile<U>(vec, nv, next_tile + nwaves, lane, done);
        if (next_tile < ntiles) {
            const int rel = eos_rel0 - next_tile * (4 * kWave * U);
            if (eos_rel0 >= 0 && rel >= 0 && rel < 4 * kWave * U) block_eos<U>(next, rel, lane);
            if (nwaves > 1) {
                st.floor = fmaxf(st.floor, float_from_ord(sm.thr));
                st.thr = fmaxf(st.thr, st.floor);
            }
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
    // elements before the first / after the last 16-byte aligned group (rows whose
    // length or start is not a multiple of four floats): at most 3 + 3, one per lane
    if (wave == 0 && head + tail > 0) {
        const bool mine = lane < head + tail;
        const int w = lane < head ? lane : head + (nv << 2) + (lane - head);
        const float s = mine ? prev + row[w] : -INFINITY;
        u64 m = __ballot(mine && (s >= st.thr) && (w != eos_block));
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const int wl = l < head ? l : head + (nv << 2) + (l - head);
            const uint32_t sbits = (uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(s), l);
            if (cnt + 1 > kStageCap) flush_stage(st, stage, cnt, kk);
            if (lane == 0) stage[cnt] = make_key_uniform(sbits, flat_base + (uint32_t)wl);
            cnt += 1;
        }
    }
    if (cnt > 0) flush_stage(st, stage, cnt, kk);
}

// ---------------------------------------------------------------------------
// constraint bookkeeping (Sec. 3.1): in-order phrases, one phrase under way
// ---------------------------------------------------------------------------
// Token that phrase j lets the hypothesis place now, or -1: the next token of
// the phrase under way; the first token of a phrase neither complete nor under way.
__device__ __forceinline__ int expandable_token(const MergeSmem &sm, u64 met, int ip, int iq, int j)
{
    const int o = sm.poff[j];
    if (j == ip) return sm.tok[o + iq];
    const int last = sm.poff[j + 1] - 1;
    if ((met >> last) & 1ull) return -1;
    return sm.tok[o];
}

// State after emitting w: advance the phrase under way, or unwind it and let w
// begin the lowest-index incomplete phrase that starts with w.
__device__ __forceinline__ void cons_add(const MergeSmem &sm, int P, u64 &met, int &ip, int &iq, int w)
{
    if (ip >= 0) {
        const int o = sm.poff[ip];
        if (sm.tok[o + iq] == w) {
            met |= 1ull << (o + iq);
            ++iq;
            if (o + iq == sm.poff[ip + 1]) {
                ip = -1;
                iq = 0;
            }
            return;
        }
        met &= ~(((1ull << iq) - 1ull) << o);
        ip = -1;
        iq = 0;
    }
    for (int j = 0; j < P; ++j) {
        const int o = sm.poff[j], e = sm.poff[j + 1];
        if ((met >> (e - 1)) & 1ull) continue;
        if (sm.tok[o] != w) continue;
        met |= 1ull << o;
        if (e - o > 1) {
            ip = j;
            iq = 1;
        }
        return;
    }
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
__device__ __forceinline__ int allocate_wave(int k, int C, int c, int c64, int &a64)
{
    const int lane = lane_id();
    const int base = k / (C + 1);
    const int rem = k - base * (C + 1);
    int a = (lane <= C) ? base + (lane == C ? rem : 0) : 0;
    a64 = (C == 64) ? base + rem : 0;
    if (lane > C) c = 0;
    if (C < 64) c64 = 0;

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

// sorts buf[0..n) (n a power of two) in decreasing order; all threads of the block take part
__device__ __forceinline__ void block_sort_desc(u64 *buf, int n)
{
    for (int k2 = 2; k2 <= n; k2 <<= 1) {
        for (int j = k2 >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (n >> 1); t += kBlock) {
                const int i = 2 * t - (t & (j - 1));
                const int l = i + j;
                const bool desc_block = (i & k2) == 0;
                const u64 a = buf[i], c = buf[l];
                if ((a < c) == desc_block) {
                    buf[i] = c;
                    buf[l] = a;
                }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ void merge_phase(const StepParams &p, int b, MergeSmem &sm, u64 *sortbuf)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int k = p.k, V = p.V;
    const int P = p.nphr[b];
    const int32_t *goff = p.phr_off + (size_t)b * (kMaxCons + 1);
    const int C = goff[P];

    if (tid <= P) sm.poff[tid] = goff[tid];
    if (tid < C) sm.tok[tid] = p.cons_tok[(size_t)b * kMaxCons + tid];
    if (tid <= kMaxCons) sm.cnt[tid] = 0;
    if (tid == 0) sm.nsel = 0;
    if (tid < k) {
        const size_t r = (size_t)b * k + tid;
        sm.prev[tid] = p.score_cur[r];
        sm.met[tid] = p.met_cur[r];
        sm.ipq[tid] = p.ipq_cur[r];
        sm.len[tid] = p.len_cur[r];
        sm.fin[tid] = p.fin_cur[r];
    }

    // source 1: the sentence's k best (Sec. 3.1 item 1) = top k of the union of the row lists
    u64 acc = 0;
    for (int h = wave; h < k; h += kWavesPerBlock) {
        const u64 L = p.rowlists[((size_t)b * k + h) * kWave + lane];
        if (lane == 0) sm.rb[h] = L;                  // source 3: the row's best (item 3)
        acc = merge_desc<u64>(acc, L);
    }
    sm.wl[wave][lane] = acc;
    const int ncand_max = k * (P + 2);
    int npad = kWave;
    while (npad < ncand_max) npad <<= 1;
    for (int i = tid; i < npad; i += kBlock) sortbuf[i] = 0;
    __syncthreads();
    if (wave == 0) {
        for (int w = 1; w < kWavesPerBlock; ++w) acc = merge_desc<u64>(acc, sm.wl[w][lane]);
        sm.t1[lane] = lane < k ? acc : 0ull;
    }
    __syncthreads();

    // tau = k-th best key of the sentence; 0 while fewer than k finite sums exist, in which
    // case every finite sum is among the k best already.
    const u64 tau = sm.t1[k - 1];

    // candidates, deduplicated by construction: the k best; a row's best unless among the
    // k best; an expandable constraint token (item 2) unless among the k best, equal to its
    // row's best, or offered already by a lower phrase of the same hypothesis.
    for (int i = tid; i < ncand_max; i += kBlock) {
        u64 key = 0;
        int h = 0, w = 0;
        bool valid = false;
        if (i < k) {
            key = sm.t1[i];
            valid = key != 0;
            if (valid) {
                const uint32_t flat = key_flat(key);
                h = (int)(flat / (uint32_t)V);
                w = (int)(flat - (uint32_t)h * (uint32_t)V);
            }
        } else if (i < 2 * k) {
            h = i - k;
            key = sm.rb[h];
            valid = key != 0 && tau != 0 && key < tau;
            if (valid) w = (int)(key_flat(key) - (uint32_t)h * (uint32_t)V);
        } else {
            const int q = i - 2 * k;
            h = q / P;
            const int j = q - h * P;
            const float pv = sm.prev[h];
            if (pv > -INFINITY && !sm.fin[h]) {
                const u64 met = sm.met[h];
                const int ipq = sm.ipq[h];
                const int ip = ipq < 0 ? -1 : (ipq >> 8), iq = ipq < 0 ? 0 : (ipq & 255);
                const int wj = expandable_token(sm, met, ip, iq, j);
                if (wj >= 0) {
                    bool dup = false;
                    for (int j2 = 0; j2 < j; ++j2) dup |= expandable_token(sm, met, ip, iq, j2) == wj;
                    if (!dup) {
                        const float s = pv + p.logp[((size_t)b * k + h) * (size_t)V + wj];
                        if (s > -INFINITY) {
                            key = make_key(s, (uint32_t)h * (uint32_t)V + (uint32_t)wj);
                            valid = tau != 0 && key < tau && key != sm.rb[h];
                            w = wj;
                        }
                    }
                }
            }
        }
        if (valid) {
            u64 m2 = sm.met[h];
            if (!sm.fin[h]) {
                const int ipq = sm.ipq[h];
                int ip = ipq < 0 ? -1 : (ipq >> 8), iq = ipq < 0 ? 0 : (ipq & 255);
                cons_add(sm, P, m2, ip, iq, w);
            }
            const int bank = __popcll(m2);                // bank = constraints met (Sec. 3.1)
            sortbuf[i] = pack_sel(p.met_bits, bank, (uint32_t)(key >> 32), key_flat(key));
            atomicAdd(&sm.cnt[bank], 1);
        }
    }
    __syncthreads();

    // slots per bank (Sec. 3.2) and where each bank begins in the sorted order (bank C first)
    if (wave == 0) {
        const int c = sm.cnt[lane];
        const int c64 = sm.cnt[kMaxCons];
        int a64;
        const int a = allocate_wave(k, C, c, c64, a64);
        sm.alloc[lane] = a;
        if (lane == 0) sm.alloc[kMaxCons] = a64;
        const int cc = lane <= C ? c : 0;
        const int incl = wave_inclusive_sum(cc);          // candidates in banks <= lane
        const int total63 = __builtin_amdgcn_readlane(incl, 63);
        const int c64v = C == 64 ? c64 : 0;
        sm.start[lane] = (total63 - incl) + c64v;         // candidates in higher banks
        if (lane == 0) sm.start[kMaxCons] = 0;
    }
    block_sort_desc(sortbuf, npad);                       // its barriers also publish alloc/start

    // within a bank the best alloc[bank] are taken (Sec. 3.1/3.2)
    const int sel_shift = 64 - p.met_bits;
    const u64 body_mask = p.met_bits ? ((1ull << sel_shift) - 1ull) : ~0ull;
    for (int i = tid; i < npad; i += kBlock) {
        const u64 key = sortbuf[i];
        if (key != 0) {
            const int bank = p.met_bits ? (int)(key >> sel_shift) : 0;
            if (i - sm.start[bank] < sm.alloc[bank]) {
                const int slot = atomicAdd(&sm.nsel, 1);
                sm.sel[slot] = key & body_mask;
            }
        }
    }
    __syncthreads();

    // new beam, best first (Sec. 3.1); empty slots last
    if (tid < k) {
        const int nsel = sm.nsel;
        int slot = tid;
        int token = p.pad_id, parent = -1, length = 0, ipq2 = -1;
        float score = -INFINITY;
        u64 met2 = 0;
        uint8_t flags = 2, fin2 = 0;
        if (tid < nsel) {
            const u64 mine = sm.sel[tid];
            slot = 0;
            for (int j = 0; j < nsel; ++j) slot += sm.sel[j] > mine ? 1 : 0;
            const int fb = 32 - p.met_bits;
            const uint32_t flatmask = fb >= 32 ? 0xFFFFFFFFu : ((1u << fb) - 1u);
            const uint32_t flat = flatmask - ((uint32_t)mine & flatmask);
            const uint32_t ord = (uint32_t)(mine >> fb);
            parent = (int)(flat / (uint32_t)V);
            token = (int)(flat - (uint32_t)parent * (uint32_t)V);
            score = float_from_ord(ord);
            met2 = sm.met[parent];
            const int ipq = sm.ipq[parent];
            int ip = ipq < 0 ? -1 : (ipq >> 8), iq = ipq < 0 ? 0 : (ipq & 255);
            const bool pfin = sm.fin[parent] != 0;
            if (!pfin) cons_add(sm, P, met2, ip, iq, token);
            ipq2 = ip < 0 ? -1 : ((ip << 8) | iq);
            fin2 = (pfin || token == p.eos_id) ? 1 : 0;
            length = pfin ? sm.len[parent] : sm.len[parent] + 1;
            flags = fin2;
        }
        const size_t o = (size_t)b * k + slot;
        p.score_nxt[o] = score;
        p.met_nxt[o] = met2;
        p.ipq_nxt[o] = ipq2;
        p.len_nxt[o] = length;
        p.fin_nxt[o] = fin2;
        p.hist_token[o] = token;
        p.hist_backptr[o] = parent;
        if (p.out_token) p.out_token[o] = token;
        if (p.out_backptr) p.out_backptr[o] = parent;
        if (p.out_score) p.out_score[o] = score;
        if (p.out_flags) p.out_flags[o] = flags;
    }
}

}  // namespace dba
