// libdba: C-ABI implementation (see include/dba.h) and the gfx950 kernels' entry points.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "../../include/dba.h"
#include "../../include/dba_debug.h"
#include "dba_kernels.hpp"

using namespace dba;

// ---------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------
// Stream phase of one beam row (sentence b, slot h) by one workgroup of NW waves: leaves the row's
// sorted top keys in p.rowlists and the keys of its constraint tokens in p.conskeys.
// U = 16-byte loads each lane keeps in flight per tile; FMT = element type of the log-probs.
// logp, V, k, first_step are what the first loads need; the kernels take them as leading scalar
// arguments, which the hardware hands over in registers at wave start (kernel-argument preload),
// so that the first two tiles are requested before any argument has been read from memory.
template <int U, int FMT, int NW>
__device__ __forceinline__ void stream_phase(const StepParams &p, const void *logp, int V, int k, int first_step,
                                             int b, int h, StreamSmem &sm)
{
    typedef typename Logp<FMT>::elem_t elem_t;
    const int row = b * k + h;
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    constexpr int nwaves = NW;
    const bool gatherer = wave == nwaves - 1;     // this wave also fetches the constraint tokens

    // the first two tiles of the row are requested before anything else: they need nothing of
    // the hypothesis, and the loads of the hypothesis (uniform, hence scalar loads the wave has to
    // wait for one after the other) would otherwise hold them back
    const elem_t *__restrict__ logp_row = static_cast<const elem_t *>(logp) + (size_t)row * (size_t)V;
    RowStream<U, FMT> rs;
    const bool known_empty = first_step && h != 0;   // decoder-init leaves slots 1.. empty
    if (!known_empty) rs.begin(logp_row, V, wave, nwaves);
    __builtin_amdgcn_sched_barrier(0);
    // then the hypothesis and its constraint bookkeeping (one wave, one lane per phrase)
    const float prev_ld = p.score_cur[row];
    const int fin_ld = p.fin_cur[row];
    // workgroups are dealt out round-robin over the 256 compute units, so the ones sharing a
    // compute unit differ in (row / 256): let that pick the wave (hence the SIMD) that finishes the row
    const int fin_wave = (row >> 8) & (nwaves - 1);
    const bool finisher = wave == fin_wave;
    u64 g_met = 0, g_inc = 0, g_sfl = 0, t_bucket = 0;
    int g_ipq = -1, g_nxt = -1, g_ftok = -1, g_P = 0, t_btok = -1;
    if (gatherer || finisher) {
        g_met = p.met_cur[row];
        g_inc = p.inc_cur[row];
        g_ipq = p.ipq_cur[row];
        g_nxt = p.nxt_cur[row];
        g_ftok = p.first_tok[(size_t)b * kMaxCons + lane];
    }
    if (gatherer) {
        g_P = p.nphr[b];
        g_sfl = p.same_first_lower[(size_t)b * kMaxCons + lane];
    }
    if (finisher) {
        // lane j: the phrases whose first token has low six bits j, and that token where they agree on it
        t_bucket = p.first_bucket[(size_t)b * kMaxCons + lane];
        t_btok = p.bucket_tok[(size_t)b * kMaxCons + lane];
    }

    // the row's hypothesis: wave-uniform by construction, made so for the compiler
    const float prev = __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane((int)__float_as_uint(prev_ld)));
    const int fin = __builtin_amdgcn_readfirstlane(fin_ld);
    const uint32_t code_base = (uint32_t)h << p.tok_bits;

    RowTop st;
    st.list = 0;
    st.kth = 0;
    st.floor = -INFINITY;
    st.thr = kLowestFinite;
    u64 ckey = 0;
    int parked = 0;
    if (prev > -INFINITY && !(fin & kFinFinished) && !known_empty) {
        // Alg. 2 inner loop / Sec. 3.1 item 2: the hypothesis extended by each constraint token
        // it may place now; the log-prob is one 4-byte read per token, in flight during the stream
        int cw = -1, cbank = 0;
        if (gatherer)
            cw = expandable_entry(g_P, __popcll(g_met), g_inc, g_ipq < 0 ? -1 : (g_ipq >> 8),
                                  g_ipq < 0 ? 0 : (g_ipq & 255), g_nxt, g_ftok, g_sfl, cbank);
        const float cx = cw >= 0 ? Logp<FMT>::widen_one(logp_row[cw]) : -INFINITY;
        // Sec. 3.3: no end-of-sentence before all constraints are met
        const int eos_block = (fin & kFinEosBlocked) ? p.eos_id : -1;
        parked = rs.run(prev, eos_block, code_base, k, wave, nwaves, sm, st);
        const float cs = prev + cx;
        if (cw >= 0 && cs > -INFINITY)
            ckey = pack_sel(p.met_bits, cbank, ord_from_float(cs), code_base | (uint32_t)cw);
    } else if (prev > -INFINITY && wave == 0 && lane == 0) {
        // a finished hypothesis stays on the beam: its one continuation is the pad token
        // at log-prob +0.0, score carried unchanged
        st.list = make_key(prev + 0.0f, code_base | (uint32_t)p.pad_id);
    }
    if (gatherer) {
        p.conskeys[(size_t)row * kMaxCons + lane] = ckey;
    }
    const u64 acc = finish_row(sm, st.list, parked, wave, nwaves, fin_wave);
    if (finisher) {
        // Handed on as selection keys: every listed sum with the bank it would land in - the
        // constraints met once the hypothesis has emitted that token (add(), Sec. 3.1).  Each lane
        // looks its own token up in the sentence's table of first tokens, which the lanes of this
        // wave hold (lane j = bucket j): the phrases it could begin, then the count.
        // (every lane takes every step, so that any lane's table entry can be read)
        const int nmet = __popcll(g_met);
        const bool extends = !(fin & kFinFinished) && acc != 0;      // not the carried-over key of a finished row
        const int w = extends ? (int)(key_flat(acc) & ((1u << p.tok_bits) - 1u)) : 0;
        const int same = __shfl(t_btok, w & 63, kWave);
        const u64 bucket = ((u64)(uint32_t)__shfl((int)(uint32_t)(t_bucket >> 32), w & 63, kWave) << 32) |
                           (u64)(uint32_t)__shfl((int)(uint32_t)t_bucket, w & 63, kWave);
        u64 match = (extends && same == w) ? bucket : 0;
        u64 todo = (extends && same == -2) ? bucket : 0;   // the bucket's phrases begin differently: one by one
        while (__ballot(todo != 0)) {
            const int j = todo ? __ffsll((long long)todo) - 1 : 0;
            const int first = __shfl(g_ftok, j, kWave);
            if (todo && first == w) match |= 1ull << j;
            todo &= todo - 1;
        }
        const int bank = !extends ? nmet
                                  : nmet_after(nmet, g_ipq < 0 ? -1 : (g_ipq >> 8), g_ipq < 0 ? 0 : (g_ipq & 255),
                                               w == g_nxt, match, g_inc);
        p.rowlists[(size_t)row * kWave + lane] = sel_from_rowkey(p.met_bits, bank, acc);
    }
}

// First launch of a step.  Grid: (k, B) workgroups of NW waves, one per beam row, in row
// order.  k_first = k | first_step << 16.
template <int U, int FMT, int NW>
__global__ __launch_bounds__(NW * kWave) void dba_stream_kernel(const void *logp, int V, int k_first, const StepParams p)
{
    __shared__ StreamSmem sm;
    stream_phase<U, FMT, NW>(p, logp, V, k_first & 0xFFFF, k_first >> 16, (int)blockIdx.y, (int)blockIdx.x, sm);
}

// Second launch of a step: the merge phase.  Grid: one workgroup of MW waves per sentence, each wave
// taking up to ROWS beam rows (k <= ROWS * MW).  The pointers to the row lists and the beam width
// come first: they are all the first loads need.
template <int ROWS, int MW>
__global__ __launch_bounds__(MW * kWave) void dba_merge_kernel(const u64 *rowlists, const u64 *conskeys, int k,
                                                               const StepParams p)
{
    extern __shared__ __align__(16) unsigned char dyn_smem[];
    __shared__ MergeSmem sm;
    merge_phase<ROWS, MW>(p, rowlists, conskeys, k, (int)blockIdx.x, sm, reinterpret_cast<u64 *>(dyn_smem));
}

// Reference read: the largest element of each row, one workgroup per row, with the tile order and
// the two-tiles-in-flight non-temporal 128-bit loads of the stream phase and nothing else.  Its
// duration is what this chip takes to deliver the [rows, V] tensor once; the step is compared
// with it.
__global__ __launch_bounds__(kBlock) void dba_row_max_kernel(const float *__restrict__ src, int V,
                                                             float *__restrict__ out)
{
    typedef float v4f __attribute__((ext_vector_type(4)));
    constexpr int U = 4;
    __shared__ float part[kWavesPerBlock];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const v4f *vec = reinterpret_cast<const v4f *>(src + (size_t)blockIdx.x * V);
    const int nv = V >> 2, per = kWave * U, ntiles = (nv + per - 1) / per;
    const float ninf = -__builtin_inff();
    v4f a[U], b[U];
    auto load = [&](v4f(&x)[U], int tl) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = tl * per + u * kWave + lane;
            x[u] = i < nv ? __builtin_nontemporal_load(vec + i) : v4f{ninf, ninf, ninf, ninf};
        }
    };
    float m = ninf;
    auto fold = [&](v4f(&x)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) m = fmaxf(m, fmaxf(fmaxf(x[u].x, x[u].y), fmaxf(x[u].z, x[u].w)));
    };
    int tl = wave;
    if (tl < ntiles) load(a, tl);
    if (tl + kWavesPerBlock < ntiles) load(b, tl + kWavesPerBlock);
    while (tl < ntiles) {
        fold(a);
        if (tl + 2 * kWavesPerBlock < ntiles) load(a, tl + 2 * kWavesPerBlock);
        tl += kWavesPerBlock;
        if (tl >= ntiles) break;
        fold(b);
        if (tl + 2 * kWavesPerBlock < ntiles) load(b, tl + 2 * kWavesPerBlock);
        tl += kWavesPerBlock;
    }
    for (int d = 32; d > 0; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, kWave));
    if (lane == 0) part[wave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kWavesPerBlock; ++w) m = fmaxf(m, part[w]);
        out[blockIdx.x] = m;
    }
}


// Diagnostic: the wavefront selection primitives on caller-provided keys, one wave per case.
// in: keys[128] per case, vals[64] per case.  out[0:64] = sort of keys[0:64];
// out[64:128] = merge of sort(keys[0:64]) and sort(keys[64:128]); out[128:192] = the first
// list after inserting keys[64..71] one at a time; out[192:256] = low word: the 64 greatest high
// words of both sorted lists (32-bit merge), high word: the greatest high word left out;
// fout[0:64] = sort of vals.
__global__ void dba_wave_select_kernel(int n_cases, const u64 *keys, const float *vals, u64 *out,
                                       float *fout)
{
    const int i = blockIdx.x;
    if (i >= n_cases) return;
    const int lane = lane_id();
    const u64 a = sort64_desc<u64>(keys[(size_t)i * 128 + lane]);
    const u64 b = sort64_desc<u64>(keys[(size_t)i * 128 + 64 + lane]);
    out[(size_t)i * 256 + lane] = a;
    out[(size_t)i * 256 + 64 + lane] = merge_desc<u64>(a, b);
    u64 l = a;
    for (int j = 0; j < 8; ++j) {
        const u64 x = keys[(size_t)i * 128 + 64 + j];
        l = insert_desc(l, x);
    }
    out[(size_t)i * 256 + 128 + lane] = l;
    uint32_t fell = 0;
    const uint32_t hi = merge32_desc((uint32_t)(a >> 32), (uint32_t)(b >> 32), fell);
    out[(size_t)i * 256 + 192 + lane] = ((u64)wave_max_u32(fell) << 32) | hi;
    fout[(size_t)i * 64 + lane] = float_from_ord(sort64_desc<uint32_t>(ord_from_float(vals[(size_t)i * 64 + lane])));
}

// decoder-init: slot 0 of every sentence is a live, empty hypothesis with score +0.0
__global__ void dba_init_state_kernel(int B, int k, const int32_t *phr_off, const int32_t *nphr, float *score,
                                      u64 *met, int32_t *ipq, int32_t *len, uint8_t *fin, u64 *inc,
                                      int32_t *nxt, uint8_t *all_finished, BestCompleted *best)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B * k) {
        const int b = i / k, h = i - b * k;
        const int P = nphr[b];
        const int C = phr_off[(size_t)b * (kMaxCons + 1) + P];
        score[i] = h == 0 ? 0.0f : -INFINITY;
        met[i] = 0;
        ipq[i] = -1;
        len[i] = 0;
        fin[i] = (uint8_t)((h == 0 && C > 0) ? kFinEosBlocked : 0);
        inc[i] = (h == 0 && P > 0) ? (P == 64 ? ~0ull : ((1ull << P) - 1ull)) : 0ull;
        nxt[i] = -1;
    }
    if (i < B) {
        all_finished[i] = 0;
        BestCompleted none = {};
        best[i] = none;
    }
}

// End of decoding (Sec. 3.3, length normalisation of Sec. 4): one thread per sentence.
// best != null: the record of the best completed hypothesis seen on any beam decides, if there is one.
__global__ void dba_finalize_kernel(int B, int k, int T, int N, int pad_id, int normalized,
                                    const int32_t *hist_token, const int32_t *hist_backptr,
                                    const float *score, const u64 *met, const int32_t *len,
                                    const uint8_t *fin, const BestCompleted *best_rec, int32_t *out_tokens,
                                    int32_t *out_len, float *out_score, int32_t *out_status)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int32_t *toks = out_tokens + (size_t)b * N;
    for (int i = 0; i < N; ++i) toks[i] = pad_id;
    out_len[b] = 0;
    out_score[b] = -INFINITY;
    out_status[b] = 0;
    if (T < 1) return;
    if (best_rec && best_rec[b].have) {
        const BestCompleted r = best_rec[b];
        out_status[b] = 1;
        out_len[b] = r.len;
        out_score[b] = r.score;
        int slot = r.slot;
        for (int t = r.step; t >= 0; --t) {
            const size_t at = ((size_t)t * B + b) * k + slot;
            if (t < r.len && t < N) toks[t] = hist_token[at];
            slot = hist_backptr[at];
        }
        return;
    }
    const size_t o = (size_t)b * k;
    int best = -1;
    float bestq = 0.0f;
    for (int h = 0; h < k; ++h) {
        if (!(score[o + h] > -INFINITY) || !(fin[o + h] & kFinFinished)) continue;
        // per-word score; already held by the beam when completed hypotheses are stored that way
        const float q = normalized ? score[o + h] : __fdiv_rn(score[o + h], (float)len[o + h]);
        if (best < 0 || q > bestq) {
            best = h;
            bestq = q;
        }
    }
    if (best >= 0) {
        out_status[b] = 1;
    } else {
        int bestn = -1;
        for (int h = 0; h < k; ++h) {
            if (!(score[o + h] > -INFINITY)) continue;
            const int n = __popcll(met[o + h]);
            if (best < 0 || n > bestn || (n == bestn && score[o + h] > score[o + best])) {
                best = h;
                bestn = n;
            }
        }
        if (best < 0) return;
    }
    const int L = len[o + best];
    out_len[b] = L;
    out_score[b] = score[o + best];
    int slot = best;
    for (int t = T - 1; t >= 0; --t) {
        const size_t r = ((size_t)t * B + b) * k + slot;
        if (t < L && t < N) toks[t] = hist_token[r];
        slot = hist_backptr[r];
    }
}

// Diagnostic: the allocation of Sec. 3.2 alone, one wavefront per case.
__global__ void dba_allocate_kernel(int n_cases, int adjust, const int32_t *kk, const int32_t *CC,
                                    const int32_t *cnt, int32_t *alloc)
{
    const int i = blockIdx.x;
    if (i >= n_cases) return;
    const int lane = lane_id();
    const int C = CC[i];
    const int c = cnt[(size_t)i * 65 + lane];
    const int c64 = cnt[(size_t)i * 65 + 64];
    int a64;
    const int a = allocate_wave(kk[i], C, c, c64, a64, adjust != 0);
    alloc[(size_t)i * 65 + lane] = lane <= C ? a : 0;
    if (lane == 0) alloc[(size_t)i * 65 + 64] = C == 64 ? a64 : 0;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
namespace {

thread_local char g_init_error[256] = "";

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    size_t score[2], met[2], ipq[2], len[2], fin[2], inc[2], nxt[2];
    size_t cons_tok, phr_off, nphr, ftok, sfl, bloom, btok, rowlists, conskeys;
    size_t hist_token, hist_backptr;
    size_t fin_tokens, fin_len, fin_score, fin_status, all_finished, best;
    size_t total;
};

Layout make_layout(size_t B, size_t k, size_t N)
{
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    for (int i = 0; i < 2; ++i) {
        L.score[i] = take(B * k * sizeof(float));
        L.met[i] = take(B * k * sizeof(u64));
        L.ipq[i] = take(B * k * sizeof(int32_t));
        L.len[i] = take(B * k * sizeof(int32_t));
        L.fin[i] = take(B * k);
        L.inc[i] = take(B * k * sizeof(u64));
        L.nxt[i] = take(B * k * sizeof(int32_t));
    }
    L.cons_tok = take(B * kMaxCons * sizeof(int32_t));
    L.phr_off = take(B * (kMaxCons + 1) * sizeof(int32_t));
    L.nphr = take(B * sizeof(int32_t));
    L.ftok = take(B * kMaxCons * sizeof(int32_t));
    L.sfl = take(B * kMaxCons * sizeof(u64));
    L.bloom = take(B * kMaxCons * sizeof(u64));
    L.btok = take(B * kMaxCons * sizeof(int32_t));
    L.rowlists = take(B * k * kWave * sizeof(u64));
    L.conskeys = take(B * k * kMaxCons * sizeof(u64));
    L.hist_token = take(N * B * k * sizeof(int32_t));
    L.hist_backptr = take(N * B * k * sizeof(int32_t));
    L.fin_tokens = take(B * N * sizeof(int32_t));
    L.fin_len = take(B * sizeof(int32_t));
    L.fin_score = take(B * sizeof(float));
    L.fin_status = take(B * sizeof(int32_t));
    L.all_finished = take(B);
    L.best = take(B * sizeof(BestCompleted));
    L.total = off;
    return L;
}

int bits_for(int v)   // bits needed to hold values 0..v
{
    int n = 0;
    while ((1 << n) <= v) ++n;
    return n;
}

}  // namespace

// ---------------------------------------------------------------------------
// scratch owned by the library, for dba_step_noalloc
// ---------------------------------------------------------------------------
// The two arrays that pass a step's results from its first launch to its second (every row's list
// and its constraint keys, 64 keys of 8 bytes each) for up to DBA_NOALLOC_MAX_ROWS beam rows: 8 MiB,
// present once on every GPU the library runs on, until the process ends.
constexpr size_t kStaticRows = DBA_NOALLOC_MAX_ROWS;
constexpr size_t kStaticListBytes = kStaticRows * kWave * sizeof(u64);
constexpr size_t kStaticScratchBytes = kStaticListBytes + kStaticRows * kMaxCons * sizeof(u64);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each GPU (its name is a host-side stand-in)
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device: asked for once per device, kept afterwards.
hipError_t static_scratch(void **out)
{
    *out = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct dba_ctx {
    int B, k, V, N, eos_id, pad_id;
    int met_bits;
    int tok_bits;
    int max_phrases;
    int steps;
    int adjust;                         // DBA_OPT_ADJUSTMENT
    int normalize;                      // DBA_OPT_NORMALIZE_FINISHED
    float prune;                        // DBA_OPT_PRUNE_THRESHOLD (< 0: off)
    int track;                          // DBA_OPT_TRACK_COMPLETED
    int merge_waves;                    // DBA_OPT_MERGE_WAVES (0: chosen here)
    int device;                         // the device that was current at dba_init
    unsigned char *lib_scratch;         // this device's copy of the library's own scratch (null: not resolved)
    size_t dyn_smem;
    unsigned char *ws;
    Layout L;
    hipStream_t stream;
    char err[256];
};

namespace {

int fail(dba_ctx *ctx, int code, const char *fmt, ...)
{
    char *dst = ctx ? ctx->err : g_init_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return code;
}

bool shape_ok(int B, int k, int V, int N, int max_cons)
{
    return B >= 1 && B <= 65535 && k >= 1 && k <= DBA_MAX_BEAM && V >= 1 && N >= 1 && k <= V && max_cons >= 0 &&
           max_cons <= DBA_MAX_CONS_TOKENS;
}

template <typename T>
T *at(dba_ctx *c, size_t off)
{
    return reinterpret_cast<T *>(c->ws + off);
}

}  // namespace

extern "C" {

DBA_API size_t dba_workspace_bytes(int B, int k, int V, int N, int max_cons_tokens)
{
    if (!shape_ok(B, k, V, N, max_cons_tokens)) return 0;
    return make_layout((size_t)B, (size_t)k, (size_t)N).total;
}

// dba_init proper; may throw std::bad_alloc from its host tables (caught by dba_init)
static int init_impl(dba_ctx **out, int B, int k, int V, int N, int eos_id, int pad_id,
                     const int32_t *cons_tokens, const int32_t *phrase_offsets,
                     const int32_t *sent_offsets, void *workspace_dev, size_t workspace_bytes,
                     void *hip_stream)
{
    if (!out) return fail(nullptr, DBA_EINVAL, "dba_init: out is NULL");
    *out = nullptr;
    if (!shape_ok(B, k, V, N, 0))
        return fail(nullptr, DBA_EINVAL,
                    "dba_init: need 1 <= B <= 65535, V,N >= 1 and 1 <= k <= %d, k <= V (got B=%d k=%d V=%d N=%d)",
                    DBA_MAX_BEAM, B, k, V, N);
    if (eos_id < 0 || eos_id >= V || pad_id < 0 || pad_id >= V || eos_id == pad_id)
        return fail(nullptr, DBA_EINVAL, "dba_init: eos_id/pad_id must be distinct ids in [0,V)");
    if (!sent_offsets || !phrase_offsets)
        return fail(nullptr, DBA_EINVAL, "dba_init: sent_offsets / phrase_offsets is NULL");
    if (!workspace_dev) return fail(nullptr, DBA_EINVAL, "dba_init: workspace_dev is NULL");
    if (reinterpret_cast<uintptr_t>(workspace_dev) % 256 != 0)
        return fail(nullptr, DBA_EINVAL, "dba_init: workspace_dev must be 256-byte aligned");

    // constraints -> fixed-stride per-sentence tables
    if (sent_offsets[0] != 0 || phrase_offsets[0] != 0)
        return fail(nullptr, DBA_EINVAL, "dba_init: offsets must start at 0");
    // sent_offsets[B] is the length of phrase_offsets minus one: nothing beyond it is read
    for (int b = 0; b < B; ++b)
        if (sent_offsets[b + 1] < sent_offsets[b])
            return fail(nullptr, DBA_EINVAL, "dba_init: sent_offsets decreases at %d", b);
    std::vector<int32_t> tok((size_t)B * kMaxCons, 0), off((size_t)B * (kMaxCons + 1), 0), nph(B, 0);
    std::vector<u64> sfl((size_t)B * kMaxCons, 0), bloom((size_t)B * kMaxCons, 0);
    std::vector<int32_t> ftok((size_t)B * kMaxCons, -1), btok((size_t)B * kMaxCons, -1);
    int max_tokens = 0, max_phrases = 0;
    for (int b = 0; b < B; ++b) {
        const int p0 = sent_offsets[b], p1 = sent_offsets[b + 1];
        const int t0 = phrase_offsets[p0];
        int n = 0;
        for (int p = p0; p < p1; ++p) {
            const int a = phrase_offsets[p], e = phrase_offsets[p + 1];
            if (e <= a) return fail(nullptr, DBA_EINVAL, "dba_init: phrase %d is empty or offsets decrease", p);
            if (a - t0 != n)
                return fail(nullptr, DBA_EINVAL, "dba_init: phrase offsets of sentence %d are not contiguous", b);
            if (n + (e - a) > DBA_MAX_CONS_TOKENS)
                return fail(nullptr, DBA_EINVAL, "dba_init: sentence %d has more than %d constraint tokens", b,
                            DBA_MAX_CONS_TOKENS);
            if (!cons_tokens) return fail(nullptr, DBA_EINVAL, "dba_init: cons_tokens is NULL");
            off[(size_t)b * (kMaxCons + 1) + (p - p0)] = n;
            for (int i = a; i < e; ++i) {
                const int w = cons_tokens[i];
                if (w < 0 || w >= V)
                    return fail(nullptr, DBA_EINVAL, "dba_init: constraint token %d outside [0,V)", w);
                if (w == eos_id || w == pad_id)
                    return fail(nullptr, DBA_EINVAL, "dba_init: eos_id/pad_id cannot be a constraint token");
                tok[(size_t)b * kMaxCons + n++] = w;
            }
        }
        off[(size_t)b * (kMaxCons + 1) + (p1 - p0)] = n;
        nph[b] = p1 - p0;
        // lookup aids for the kernels (layout only): which lower phrases share a phrase's first
        // token; the phrases bucketed by the low six bits of their first token; and that token
        // itself where all phrases of a bucket begin alike (-1 empty bucket, -2 they differ)
        for (int j = 0; j < p1 - p0; ++j) {
            const int fj = tok[(size_t)b * kMaxCons + off[(size_t)b * (kMaxCons + 1) + j]];
            ftok[(size_t)b * kMaxCons + j] = fj;
            bloom[(size_t)b * kMaxCons + (fj & 63)] |= 1ull << j;
            int32_t &bt = btok[(size_t)b * kMaxCons + (fj & 63)];
            bt = bt == -1 ? fj : (bt == fj ? fj : -2);
            for (int j2 = 0; j2 < j; ++j2)
                if (tok[(size_t)b * kMaxCons + off[(size_t)b * (kMaxCons + 1) + j2]] == fj)
                    sfl[(size_t)b * kMaxCons + j] |= 1ull << j2;
        }
        if (n > max_tokens) max_tokens = n;
        if (p1 - p0 > max_phrases) max_phrases = p1 - p0;
    }
    // a coordinate is (slot << tok_bits) | token; with the bank it must fit the 32 bits the
    // selection key has beside the score
    const int met_bits = bits_for(max_tokens);
    const int tok_bits = bits_for(V - 1) < 1 ? 1 : bits_for(V - 1);
    const int slot_bits = bits_for(k - 1);
    if (met_bits + slot_bits + tok_bits > 32 || tok_bits > 24)
        return fail(nullptr, DBA_EINVAL,
                    "dba_init: bits(k-1)=%d + bits(V-1)=%d + bits(max constraint tokens)=%d exceed the 32-bit "
                    "coordinate field of the selection key (or V > 2^24)", slot_bits, tok_bits, met_bits);

    const Layout L = make_layout((size_t)B, (size_t)k, (size_t)N);
    if (workspace_bytes < L.total)
        return fail(nullptr, DBA_ENOMEM, "dba_init: workspace has %zu bytes, %zu needed", workspace_bytes, L.total);

    dba_ctx *c = new (std::nothrow) dba_ctx;
    if (!c) return fail(nullptr, DBA_ENOMEM, "dba_init: out of host memory");
    memset(c, 0, sizeof *c);
    c->B = B; c->k = k; c->V = V; c->N = N; c->eos_id = eos_id; c->pad_id = pad_id;
    c->met_bits = met_bits;
    c->tok_bits = tok_bits;
    c->max_phrases = max_phrases;
    c->steps = 0;
    c->ws = static_cast<unsigned char *>(workspace_dev);
    c->L = L;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->adjust = 1;
    c->normalize = 0;
    c->prune = -1.0f;
    c->track = 0;
    c->merge_waves = 0;
    c->device = -1;
    (void)hipGetDevice(&c->device);
    void *own = nullptr;
    (void)static_scratch(&own);          // dba_step_noalloc asks again (and reports) if this failed
    c->lib_scratch = static_cast<unsigned char *>(own);
    // candidates of one sentence: at most k best + k row bests + k * phrases constraint tokens,
    // in whole chunks of 64 keys (at most 4224 keys = 33 KB of LDS)
    const int ncand_max = (k * (max_phrases + 2) + kWave - 1) / kWave * kWave;
    c->dyn_smem = (size_t)ncand_max * sizeof(u64);

    hipError_t e;
    e = hipMemcpyAsync(at<int32_t>(c, L.cons_tok), tok.data(), tok.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(at<int32_t>(c, L.phr_off), off.data(), off.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(at<int32_t>(c, L.nphr), nph.data(), nph.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(at<int32_t>(c, L.ftok), ftok.data(), ftok.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(at<u64>(c, L.sfl), sfl.data(), sfl.size() * 8, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(at<u64>(c, L.bloom), bloom.data(), bloom.size() * 8, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(at<int32_t>(c, L.btok), btok.data(), btok.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) {
        const int n = B * k;
        dba_init_state_kernel<<<(n + 255) / 256, 256, 0, c->stream>>>(
            B, k, at<int32_t>(c, L.phr_off), at<int32_t>(c, L.nphr), at<float>(c, L.score[0]),
            at<u64>(c, L.met[0]), at<int32_t>(c, L.ipq[0]), at<int32_t>(c, L.len[0]),
            at<uint8_t>(c, L.fin[0]), at<u64>(c, L.inc[0]), at<int32_t>(c, L.nxt[0]),
            at<uint8_t>(c, L.all_finished), at<BestCompleted>(c, L.best));
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);   // host tables are freed on return
    if (e != hipSuccess) {
        const int rc = fail(nullptr, DBA_EHIP, "dba_init: HIP error: %s", hipGetErrorString(e));
        delete c;
        return rc;
    }
    *out = c;
    return DBA_OK;
}

DBA_API int dba_init(dba_ctx **out, int B, int k, int V, int N, int eos_id, int pad_id,
             const int32_t *cons_tokens, const int32_t *phrase_offsets,
             const int32_t *sent_offsets, void *workspace_dev, size_t workspace_bytes,
             void *hip_stream)
{
    try {
        return init_impl(out, B, k, V, N, eos_id, pad_id, cons_tokens, phrase_offsets, sent_offsets,
                         workspace_dev, workspace_bytes, hip_stream);
    } catch (...) {                                        // nothing crosses the C boundary
        if (out) *out = nullptr;
        return fail(nullptr, DBA_ENOMEM, "dba_init: out of host memory");
    }
}

DBA_API int dba_step(dba_ctx *c, const float *logp_dev, int32_t *out_token_dev, int32_t *out_backptr_dev,
             float *out_score_dev, uint8_t *out_flags_dev)
{
    return dba_step_fmt(c, logp_dev, DBA_LOGP_F32, out_token_dev, out_backptr_dev, out_score_dev, out_flags_dev);
}

// One step.  own_scratch: the row lists and constraint keys go through the library's own scratch
// (given here as its device address) instead of the workspace.
static int step_impl(dba_ctx *c, const void *logp_dev, int logp_format, int32_t *out_token_dev,
                     int32_t *out_backptr_dev, float *out_score_dev, uint8_t *out_flags_dev,
                     unsigned char *own_scratch)
{
    if (!c) return DBA_EINVAL;
    if (!logp_dev) return fail(c, DBA_EINVAL, "dba_step: logp_dev is NULL");
    if (logp_format != DBA_LOGP_F32 && logp_format != DBA_LOGP_F16 && logp_format != DBA_LOGP_BF16)
        return fail(c, DBA_EINVAL, "dba_step: unknown log-prob format %d", logp_format);
    const unsigned elem = logp_format == DBA_LOGP_F32 ? 4u : 2u;
    if (reinterpret_cast<uintptr_t>(logp_dev) % elem != 0)
        return fail(c, DBA_EINVAL, "dba_step: logp_dev must be aligned to its element size (%u bytes)", elem);
    if (c->steps >= c->N) return fail(c, DBA_ESTATE, "dba_step: all N=%d steps have been taken", c->N);

    const int cur = c->steps & 1, nxt = cur ^ 1;
    const Layout &L = c->L;
    StepParams p;
    p.B = c->B; p.k = c->k; p.V = c->V;
    p.eos_id = c->eos_id; p.pad_id = c->pad_id;
    p.met_bits = c->met_bits;
    p.tok_bits = c->tok_bits;
    p.first_step = c->steps == 0 ? 1 : 0;
    p.cand_cap = (int)(c->dyn_smem / sizeof(u64));
    p.adjust = c->adjust;
    p.normalize = c->normalize;
    p.prune = c->prune;
    p.track = c->track;
    p.step = c->steps;
    p.logp = logp_dev;
    p.score_cur = at<float>(c, L.score[cur]);
    p.met_cur = at<u64>(c, L.met[cur]);
    p.ipq_cur = at<int32_t>(c, L.ipq[cur]);
    p.len_cur = at<int32_t>(c, L.len[cur]);
    p.fin_cur = at<uint8_t>(c, L.fin[cur]);
    p.inc_cur = at<u64>(c, L.inc[cur]);
    p.nxt_cur = at<int32_t>(c, L.nxt[cur]);
    p.score_nxt = at<float>(c, L.score[nxt]);
    p.met_nxt = at<u64>(c, L.met[nxt]);
    p.ipq_nxt = at<int32_t>(c, L.ipq[nxt]);
    p.len_nxt = at<int32_t>(c, L.len[nxt]);
    p.fin_nxt = at<uint8_t>(c, L.fin[nxt]);
    p.inc_nxt = at<u64>(c, L.inc[nxt]);
    p.nxt_nxt = at<int32_t>(c, L.nxt[nxt]);
    p.cons_tok = at<int32_t>(c, L.cons_tok);
    p.phr_off = at<int32_t>(c, L.phr_off);
    p.nphr = at<int32_t>(c, L.nphr);
    p.first_tok = at<int32_t>(c, L.ftok);
    p.same_first_lower = at<u64>(c, L.sfl);
    p.first_bucket = at<u64>(c, L.bloom);
    p.bucket_tok = at<int32_t>(c, L.btok);
    p.rowlists = own_scratch ? reinterpret_cast<u64 *>(own_scratch) : at<u64>(c, L.rowlists);
    p.conskeys = own_scratch ? reinterpret_cast<u64 *>(own_scratch + kStaticListBytes) : at<u64>(c, L.conskeys);
    p.out_token = out_token_dev;
    p.out_backptr = out_backptr_dev;
    p.out_score = out_score_dev;
    p.out_flags = out_flags_dev;
    const size_t hrow = (size_t)c->steps * c->B * c->k;
    p.hist_token = at<int32_t>(c, L.hist_token) + hrow;
    p.hist_backptr = at<int32_t>(c, L.hist_backptr) + hrow;
    p.all_finished = at<uint8_t>(c, L.all_finished);
    p.best = at<BestCompleted>(c, L.best);

    // one workgroup per beam row, 4 loads of 16 bytes per lane and tile, two 4 KB tiles in flight per wave: at
    // 1280 rows of four waves the 1024 SIMDs are filled five deep (measured best on MI355X at V = 32000)
    const dim3 grid((unsigned)c->k, (unsigned)c->B);      // row order: slot fastest
    const int kf = p.k | (p.first_step << 16);
    {
        // Waves per beam row (measured on MI355X, fp32 and 16-bit inputs, 10 to 8192 rows): eight where the
        // grid cannot fill the chip by itself (at most two rows per compute unit) and a row has work for
        // them, and where rows are long (from 160 KB on: the floor then rests on a larger share of the
        // row and fewer sums are looked at closely); four otherwise - with rows of 64-128 KB and
        // thousands of them, twice the workgroups per compute unit stream faster than twice the waves.
        const size_t row_bytes = (size_t)c->V * elem;
        const int stream_waves =
            (((size_t)c->B * c->k <= 512 && row_bytes >= 32768) || row_bytes >= 163840) ? 8 : 4;
        const dim3 sblock((unsigned)(stream_waves * kWave));
        if (stream_waves == 8) {
            switch (logp_format) {
                case DBA_LOGP_F16: dba_stream_kernel<kTileLoads, kFmtF16, 8><<<grid, sblock, 0, c->stream>>>(p.logp, p.V, kf, p); break;
                case DBA_LOGP_BF16: dba_stream_kernel<kTileLoads, kFmtBF16, 8><<<grid, sblock, 0, c->stream>>>(p.logp, p.V, kf, p); break;
                default: dba_stream_kernel<kTileLoads, kFmtF32, 8><<<grid, sblock, 0, c->stream>>>(p.logp, p.V, kf, p); break;
            }
        } else {
            switch (logp_format) {
                case DBA_LOGP_F16: dba_stream_kernel<kTileLoads, kFmtF16, 4><<<grid, sblock, 0, c->stream>>>(p.logp, p.V, kf, p); break;
                case DBA_LOGP_BF16: dba_stream_kernel<kTileLoads, kFmtBF16, 4><<<grid, sblock, 0, c->stream>>>(p.logp, p.V, kf, p); break;
                default: dba_stream_kernel<kTileLoads, kFmtF32, 4><<<grid, sblock, 0, c->stream>>>(p.logp, p.V, kf, p); break;
            }
        }
        // The merge phase is compiled for (rows per wave, waves): the beam rows of a sentence are dealt out to
        // the waves of its workgroup.  Unless the caller fixes the waves: four waves of four rows up to k = 16;
        // from there on eight waves (of four rows up to k = 32, of eight beyond): fewer lists per wave to merge
        // and to scan, a wave of its own for every chunk of candidates, at the price of a deeper tree where the
        // waves' lists are joined (measured on MI355X, one decode: 6.2 / 6.5 us with four / eight waves at
        // k = 10, 7.7 / 7.0 at k = 20, 19.3 / 14.6 at k = 64).
        const dim3 mgrid((unsigned)c->B);
        const dim3 mblock8(8 * kWave), mblock4(4 * kWave);
        const int mw = c->merge_waves ? c->merge_waves : (c->k <= 16 ? 4 : 8);
        if (mw == 4) {
            if (c->k <= 16) dba_merge_kernel<4, 4><<<mgrid, mblock4, c->dyn_smem, c->stream>>>(p.rowlists, p.conskeys, p.k, p);
            else if (c->k <= 32) dba_merge_kernel<8, 4><<<mgrid, mblock4, c->dyn_smem, c->stream>>>(p.rowlists, p.conskeys, p.k, p);
            else dba_merge_kernel<16, 4><<<mgrid, mblock4, c->dyn_smem, c->stream>>>(p.rowlists, p.conskeys, p.k, p);
        } else {
            if (c->k <= 32) dba_merge_kernel<4, 8><<<mgrid, mblock8, c->dyn_smem, c->stream>>>(p.rowlists, p.conskeys, p.k, p);
            else dba_merge_kernel<8, 8><<<mgrid, mblock8, c->dyn_smem, c->stream>>>(p.rowlists, p.conskeys, p.k, p);
        }
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, DBA_EHIP, "dba_step: launch failed: %s", hipGetErrorString(e));
    c->steps += 1;
    return DBA_OK;
}

DBA_API int dba_step_fmt(dba_ctx *c, const void *logp_dev, int logp_format, int32_t *out_token_dev,
                         int32_t *out_backptr_dev, float *out_score_dev, uint8_t *out_flags_dev)
{
    return step_impl(c, logp_dev, logp_format, out_token_dev, out_backptr_dev, out_score_dev, out_flags_dev,
                     nullptr);
}

DBA_API int dba_step_noalloc(dba_ctx *c, const void *logp_dev, int logp_format, int32_t *out_token_dev,
                             int32_t *out_backptr_dev, float *out_score_dev, uint8_t *out_flags_dev)
{
    if (!c) return DBA_EINVAL;
    if ((size_t)c->B * (size_t)c->k > kStaticRows)
        return fail(c, DBA_EINVAL,
                    "dba_step_noalloc: B*k = %zu beam rows exceed the %zu rows (DBA_NOALLOC_MAX_ROWS) the "
                    "library's own scratch holds; use dba_step / dba_step_fmt",
                    (size_t)c->B * (size_t)c->k, kStaticRows);
    if (!c->lib_scratch) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev != c->device)
            return fail(c, DBA_ESTATE, "dba_step_noalloc: the device of dba_init (%d) must be current", c->device);
        void *own = nullptr;
        const hipError_t e = static_scratch(&own);
        if (e != hipSuccess)
            return fail(c, DBA_EHIP, "dba_step_noalloc: the library's scratch has no device address: %s",
                        hipGetErrorString(e));
        c->lib_scratch = static_cast<unsigned char *>(own);
    }
    return step_impl(c, logp_dev, logp_format, out_token_dev, out_backptr_dev, out_score_dev, out_flags_dev,
                     c->lib_scratch);
}

DBA_API int dba_finalize(dba_ctx *c, int32_t *out_tokens_host, int32_t *out_len_host, float *out_score_host,
                 int32_t *out_status_host)
{
    if (!c) return DBA_EINVAL;
    if (!out_tokens_host || !out_len_host || !out_score_host || !out_status_host)
        return fail(c, DBA_EINVAL, "dba_finalize: an output pointer is NULL");
    const Layout &L = c->L;
    const int cur = c->steps & 1;
    dba_finalize_kernel<<<(c->B + 63) / 64, 64, 0, c->stream>>>(
        c->B, c->k, c->steps, c->N, c->pad_id, c->normalize, at<int32_t>(c, L.hist_token),
        at<int32_t>(c, L.hist_backptr),
        at<float>(c, L.score[cur]), at<u64>(c, L.met[cur]), at<int32_t>(c, L.len[cur]),
        at<uint8_t>(c, L.fin[cur]), c->track ? at<BestCompleted>(c, L.best) : nullptr,
        at<int32_t>(c, L.fin_tokens), at<int32_t>(c, L.fin_len),
        at<float>(c, L.fin_score), at<int32_t>(c, L.fin_status));
    hipError_t e = hipGetLastError();
    const size_t B = (size_t)c->B;
    if (e == hipSuccess)
        e = hipMemcpyAsync(out_tokens_host, at<int32_t>(c, L.fin_tokens), B * c->N * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(out_len_host, at<int32_t>(c, L.fin_len), B * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(out_score_host, at<float>(c, L.fin_score), B * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(out_status_host, at<int32_t>(c, L.fin_status), B * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail(c, DBA_EHIP, "dba_finalize: HIP error: %s", hipGetErrorString(e));
    return DBA_OK;
}

DBA_API int dba_get_state(dba_ctx *c, float *score_host, uint64_t *met_mask_host, int32_t *inprog_phrase_host,
                  int32_t *inprog_pos_host, int32_t *length_host, uint8_t *flags_host)
{
    if (!c) return DBA_EINVAL;
    const Layout &L = c->L;
    const int cur = c->steps & 1;
    const size_t n = (size_t)c->B * c->k;
    // one host block for the three arrays this call decodes: n floats, n ints, n bytes
    unsigned char *tmp = static_cast<unsigned char *>(malloc(n * 9 + 16));
    if (!tmp) return fail(c, DBA_ENOMEM, "dba_get_state: out of host memory");
    struct Free {
        unsigned char *p;
        ~Free() { free(p); }
    } guard{tmp};
    float *score = reinterpret_cast<float *>(tmp);
    int32_t *ipq = reinterpret_cast<int32_t *>(tmp + n * 4);
    uint8_t *fin = tmp + n * 8;
    hipError_t e = hipMemcpyAsync(score, at<float>(c, L.score[cur]), n * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(ipq, at<int32_t>(c, L.ipq[cur]), n * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(fin, at<uint8_t>(c, L.fin[cur]), n, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess && met_mask_host)
        e = hipMemcpyAsync(met_mask_host, at<u64>(c, L.met[cur]), n * 8, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess && length_host)
        e = hipMemcpyAsync(length_host, at<int32_t>(c, L.len[cur]), n * 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail(c, DBA_EHIP, "dba_get_state: HIP error: %s", hipGetErrorString(e));
    for (size_t i = 0; i < n; ++i) {
        if (score_host) score_host[i] = score[i];
        if (inprog_phrase_host) inprog_phrase_host[i] = ipq[i] < 0 ? -1 : (ipq[i] >> 8);
        if (inprog_pos_host) inprog_pos_host[i] = ipq[i] < 0 ? 0 : (ipq[i] & 255);
        if (flags_host)
            flags_host[i] = (uint8_t)(((fin[i] & kFinFinished) ? DBA_FLAG_FINISHED : 0) | (score[i] > -INFINITY ? 0 : DBA_FLAG_DEAD));
    }
    return DBA_OK;
}

DBA_API int dba_steps_done(const dba_ctx *c) { return c ? c->steps : DBA_EINVAL; }

DBA_API int dba_set_option(dba_ctx *c, int option, double value)
{
    if (!c) return DBA_EINVAL;
    if (c->steps != 0) return fail(c, DBA_ESTATE, "dba_set_option: options are fixed once the first step is taken");
    if (value != value) return fail(c, DBA_EINVAL, "dba_set_option: the value is not a number");
    switch (option) {
        case DBA_OPT_ADJUSTMENT: c->adjust = value != 0.0 ? 1 : 0; return DBA_OK;
        case DBA_OPT_NORMALIZE_FINISHED: c->normalize = value != 0.0 ? 1 : 0; return DBA_OK;
        case DBA_OPT_PRUNE_THRESHOLD: c->prune = value < 0.0 ? -1.0f : (float)value; return DBA_OK;
        case DBA_OPT_TRACK_COMPLETED: c->track = value != 0.0 ? 1 : 0; return DBA_OK;
        case DBA_OPT_MERGE_WAVES:
            if (value != 0.0 && value != 4.0 && value != 8.0)
                return fail(c, DBA_EINVAL, "dba_set_option: DBA_OPT_MERGE_WAVES takes 0, 4 or 8");
            c->merge_waves = (int)value;
            return DBA_OK;
        default: return fail(c, DBA_EINVAL, "dba_set_option: unknown option %d", option);
    }
}

DBA_API int dba_get_finished(dba_ctx *c, uint8_t *all_finished_host)
{
    if (!c) return DBA_EINVAL;
    if (!all_finished_host) return fail(c, DBA_EINVAL, "dba_get_finished: the output pointer is NULL");
    hipError_t e = hipMemcpyAsync(all_finished_host, at<uint8_t>(c, c->L.all_finished), (size_t)c->B,
                                  hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail(c, DBA_EHIP, "dba_get_finished: HIP error: %s", hipGetErrorString(e));
    return DBA_OK;
}

DBA_API void dba_destroy(dba_ctx *c) { delete c; }

DBA_API const char *dba_last_error(const dba_ctx *c) { return c ? c->err : g_init_error; }

DBA_API int dba_debug_allocate(int n_cases, int adjust, const int32_t *k_host, const int32_t *C_host, const int32_t *cnt_host,
                       int32_t *alloc_host, void *scratch_dev, size_t scratch_bytes, void *hip_stream)
{
    if (n_cases < 1 || !k_host || !C_host || !cnt_host || !alloc_host || !scratch_dev)
        return fail(nullptr, DBA_EINVAL, "dba_debug_allocate: bad argument");
    const size_t n = (size_t)n_cases;
    if (scratch_bytes < n * 132 * 4) return fail(nullptr, DBA_ENOMEM, "dba_debug_allocate: scratch too small");
    for (size_t i = 0; i < n; ++i)
        if (k_host[i] < 1 || k_host[i] > DBA_MAX_BEAM || C_host[i] < 0 || C_host[i] > DBA_MAX_CONS_TOKENS)
            return fail(nullptr, DBA_EINVAL, "dba_debug_allocate: case %zu out of range", i);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int32_t *d_k = static_cast<int32_t *>(scratch_dev);
    int32_t *d_C = d_k + n;
    int32_t *d_cnt = d_C + n;
    int32_t *d_alloc = d_cnt + n * 65;
    hipError_t e = hipMemcpyAsync(d_k, k_host, n * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(d_C, C_host, n * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(d_cnt, cnt_host, n * 65 * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) {
        dba_allocate_kernel<<<dim3((unsigned)n_cases), dim3(kWave), 0, s>>>(n_cases, adjust, d_k, d_C, d_cnt, d_alloc);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(alloc_host, d_alloc, n * 65 * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(nullptr, DBA_EHIP, "dba_debug_allocate: HIP error: %s", hipGetErrorString(e));
    return DBA_OK;
}

DBA_API int dba_debug_wave_select(int n_cases, const uint64_t *keys_host, const float *vals_host,
                                  uint64_t *out_host, float *fout_host, void *scratch_dev,
                                  size_t scratch_bytes, void *hip_stream)
{
    if (n_cases < 1 || !keys_host || !vals_host || !out_host || !fout_host || !scratch_dev)
        return fail(nullptr, DBA_EINVAL, "dba_debug_wave_select: bad argument");
    const size_t n = (size_t)n_cases;
    if (scratch_bytes < n * (128 * 8 + 256 * 8 + 64 * 4 + 64 * 4))
        return fail(nullptr, DBA_ENOMEM, "dba_debug_wave_select: scratch too small");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    u64 *d_keys = static_cast<u64 *>(scratch_dev);
    u64 *d_out = d_keys + n * 128;
    float *d_vals = reinterpret_cast<float *>(d_out + n * 256);
    float *d_fout = d_vals + n * 64;
    hipError_t e = hipMemcpyAsync(d_keys, keys_host, n * 128 * 8, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(d_vals, vals_host, n * 64 * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) {
        dba_wave_select_kernel<<<dim3((unsigned)n_cases), dim3(kWave), 0, s>>>(n_cases, d_keys, d_vals, d_out, d_fout);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(out_host, d_out, n * 256 * 8, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipMemcpyAsync(fout_host, d_fout, n * 64 * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(nullptr, DBA_EHIP, "dba_debug_wave_select: HIP error: %s", hipGetErrorString(e));
    return DBA_OK;
}

DBA_API int dba_debug_row_max(const float *src_dev, int rows, int V, float *out_max_dev, void *hip_stream)
{
    if (!src_dev || !out_max_dev || rows < 1 || V < 4 || (V & 3))
        return fail(nullptr, DBA_EINVAL, "dba_debug_row_max: bad argument (V must be a multiple of 4)");
    if (reinterpret_cast<uintptr_t>(src_dev) & 15)
        return fail(nullptr, DBA_EINVAL, "dba_debug_row_max: src_dev must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    dba_row_max_kernel<<<dim3((unsigned)rows), dim3(kBlock), 0, s>>>(src_dev, V, out_max_dev);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(nullptr, DBA_EHIP, "dba_debug_row_max: HIP error: %s", hipGetErrorString(e));
    return DBA_OK;
}

}  // extern "C"
