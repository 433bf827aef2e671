// Wavefront-level selection primitives for gfx950 (64 lanes), registers only.
//
// A "list" is 64 keys, one per lane, sorted in decreasing order; unused places
// hold 0.  Keys are 64-bit and strictly ordered: the high word is an
// order-preserving image of an fp32 score, the low word is the complement of
// the flat coordinate h*V+w, so "greater key" means "higher score, then lower
// coordinate" - the tie rule of the step - and no two live keys are equal.
//
// Lane exchanges: DPP (quad permutes, row mirrors, wave shift) where one VALU move does it,
// ds_swizzle (the LDS crossbar, no memory access, issued outside the VALU) for the other
// patterns inside 32 lanes, and the gfx950 permlane32 swap across the wave's halves.  A
// compare-exchange stage is then one 64-bit compare and two selects on the VALU; the
// direction of each lane is a loop-invariant lane mask folded in with a scalar xor.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dba {

typedef unsigned long long u64;

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// fp32 -> u32 with the same ordering as the floats (-0.0 made +0.0 first).
__device__ __forceinline__ uint32_t ord_from_float(float s)
{
    s = s + 0.0f;
    const uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float float_from_ord(uint32_t o)
{
    const uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
    return __uint_as_float(u);
}

__device__ __forceinline__ u64 make_key(float s, uint32_t flat)
{
    return ((u64)ord_from_float(s) << 32) | (u64)(0xFFFFFFFFu - flat);
}

__device__ __forceinline__ uint32_t key_flat(u64 key) { return 0xFFFFFFFFu - (uint32_t)key; }

// Wave-uniform read of one lane's key (lane index must be wave-uniform).
__device__ __forceinline__ u64 read_lane(u64 v, int l)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((u64)hi << 32) | lo;
}

// ---- lane permutations of one 32-bit register ------------------------------
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppQuadRev = 0x1B;     // quad_perm [3,2,1,0]   lane ^ 3
constexpr int kDppWaveShr1 = 0x138;   // lane i reads lane i-1 (lane 0 reads 0)
constexpr int kDppRowMirror = 0x140;  // lane ^ 15
constexpr int kDppHalfMirror = 0x141; // lane ^ 7

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xf, 0xf, true);
}

// lane' = ((lane & 31) ^ X) inside each half of the wave
template <int X>
__device__ __forceinline__ uint32_t swizzle_xor_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (X << 10));
}

// value held by lane (lane ^ 32): the wave's halves are exchanged
__device__ __forceinline__ uint32_t xor32_u32(uint32_t v)
{
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (lane_id() & 32) ? r[0] : r[1];
}

// value held by lane (lane ^ 16): rows of 16 lanes are exchanged pairwise
__device__ __forceinline__ uint32_t xor16_valu_u32(uint32_t v)
{
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return (lane_id() & 16) ? r[0] : r[1];
}

// Two flavours of every exchange.  LL = false: the fewest VALU instructions (ds_swizzle does
// the move outside the VALU) - for code that competes for the VALU with other waves.
// LL = true: the shortest latency (DPP / permlane only, no trip through the LDS crossbar) -
// for code whose waves run alone and wait on every step.
// value held by lane (lane ^ J), J a power of two
template <int J, bool LL>
__device__ __forceinline__ uint32_t xor_lane_u32(uint32_t v)
{
    if constexpr (J == 1) return dpp_mov<kDppXor1>(v);
    else if constexpr (J == 2) return dpp_mov<kDppXor2>(v);
    else if constexpr (J == 32) return xor32_u32(v);
    else if constexpr (!LL) return swizzle_xor_u32<J>(v);
    else if constexpr (J == 4) return dpp_mov<kDppQuadRev>(dpp_mov<kDppHalfMirror>(v));
    else if constexpr (J == 8) return dpp_mov<kDppHalfMirror>(dpp_mov<kDppRowMirror>(v));
    else return xor16_valu_u32(v);
}

// value held by the mirror lane inside blocks of S lanes: lane ^ (S-1)
template <int S, bool LL>
__device__ __forceinline__ uint32_t flip_lane_u32(uint32_t v)
{
    if constexpr (S == 2) return dpp_mov<kDppXor1>(v);
    else if constexpr (S == 4) return dpp_mov<kDppQuadRev>(v);
    else if constexpr (S == 8) return dpp_mov<kDppHalfMirror>(v);
    else if constexpr (S == 16) return dpp_mov<kDppRowMirror>(v);
    else if constexpr (S == 32) return LL ? dpp_mov<kDppRowMirror>(xor16_valu_u32(v)) : swizzle_xor_u32<31>(v);
    else return LL ? dpp_mov<kDppRowMirror>(xor16_valu_u32(xor32_u32(v))) : swizzle_xor_u32<31>(xor32_u32(v));
}

// ---- compare-exchange networks (T = u64 keys or u32 order-preserving images) ---------
template <typename T, int J, bool LL>
__device__ __forceinline__ T xor_lane_t(T v)
{
    if constexpr (sizeof(T) == 8)
        return ((u64)xor_lane_u32<J, LL>((uint32_t)(v >> 32)) << 32) | xor_lane_u32<J, LL>((uint32_t)v);
    else return xor_lane_u32<J, LL>(v);
}

template <typename T, int S, bool LL>
__device__ __forceinline__ T flip_lane_t(T v)
{
    if constexpr (sizeof(T) == 8)
        return ((u64)flip_lane_u32<S, LL>((uint32_t)(v >> 32)) << 32) | flip_lane_u32<S, LL>((uint32_t)v);
    else return flip_lane_u32<S, LL>(v);
}

// half-cleaner at distance J: the lower lane of each pair keeps the greater value
template <typename T, int J, bool LL>
__device__ __forceinline__ T clean_desc(T v)
{
    const T other = xor_lane_t<T, J, LL>(v);
    const bool upper = (lane_id() & J) != 0;
    return ((v < other) != upper) ? other : v;
}

// sorts a bitonic run inside every block of S lanes, decreasing
template <typename T, int S, bool LL>
__device__ __forceinline__ T bitonic_finish_desc(T v)
{
    if constexpr (S >= 64) v = clean_desc<T, 32, LL>(v);
    if constexpr (S >= 32) v = clean_desc<T, 16, LL>(v);
    if constexpr (S >= 16) v = clean_desc<T, 8, LL>(v);
    if constexpr (S >= 8) v = clean_desc<T, 4, LL>(v);
    if constexpr (S >= 4) v = clean_desc<T, 2, LL>(v);
    if constexpr (S >= 2) v = clean_desc<T, 1, LL>(v);
    return v;
}

// merges the two decreasing halves of every block of S lanes into one decreasing block
template <typename T, int S, bool LL>
__device__ __forceinline__ T merge_halves_desc(T v)
{
    const T other = flip_lane_t<T, S, LL>(v);
    const bool upper = (lane_id() & (S >> 1)) != 0;
    v = ((v < other) != upper) ? other : v;
    return bitonic_finish_desc<T, (S >> 1), LL>(v);
}

// Full sort of one value per lane, decreasing by lane.
template <typename T, bool LL = false>
__device__ __forceinline__ T sort64_desc(T v)
{
    v = merge_halves_desc<T, 2, LL>(v);
    v = merge_halves_desc<T, 4, LL>(v);
    v = merge_halves_desc<T, 8, LL>(v);
    v = merge_halves_desc<T, 16, LL>(v);
    v = merge_halves_desc<T, 32, LL>(v);
    v = merge_halves_desc<T, 64, LL>(v);
    return v;
}

// a, b: decreasing lists.  Returns the 64 greatest of their union, decreasing.
template <typename T, bool LL = false>
__device__ __forceinline__ T merge_desc(T a, T b)
{
    const T b_rev = flip_lane_t<T, 64, LL>(b);
    return bitonic_finish_desc<T, 64, LL>(a > b_rev ? a : b_rev);   // bitonic, holds the top 64
}

// ---- 32-bit keys on the integer min/max units -------------------------------------------
// A compare-exchange stage on 32-bit keys is two min/max instructions (the lane exchange rides
// on them as a DPP operand where one DPP move does it) and a select by the lane's constant
// role: half the issue slots of the 64-bit stage above and no trip through the scalar unit.
// Equal keys are allowed.
template <int J>
__device__ __forceinline__ uint32_t clean32_desc(uint32_t v)
{
    const uint32_t o = xor_lane_u32<J, true>(v);
    const uint32_t mx = v > o ? v : o, mn = v > o ? o : v;
    return (lane_id() & J) ? mn : mx;
}

// a, b: decreasing lists of 32-bit keys.  Returns the 64 greatest of their union, decreasing;
// `fell` collects, lane by lane, the greatest key that did not make it.
__device__ __forceinline__ uint32_t merge32_desc(uint32_t a, uint32_t b, uint32_t &fell)
{
    const uint32_t b_rev = flip_lane_u32<64, true>(b);
    const uint32_t lo = a > b_rev ? b_rev : a;
    uint32_t v = a > b_rev ? a : b_rev;                  // bitonic, holds the top 64
    fell = fell > lo ? fell : lo;
    v = clean32_desc<32>(v);
    v = clean32_desc<16>(v);
    v = clean32_desc<8>(v);
    v = clean32_desc<4>(v);
    v = clean32_desc<2>(v);
    v = clean32_desc<1>(v);
    return v;
}

// greatest value of v over the wave, in every lane
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    uint32_t o;
    o = xor_lane_u32<1, true>(v); v = v > o ? v : o;
    o = xor_lane_u32<2, true>(v); v = v > o ? v : o;
    o = xor_lane_u32<4, true>(v); v = v > o ? v : o;
    o = xor_lane_u32<8, true>(v); v = v > o ? v : o;
    o = xor_lane_u32<16, true>(v); v = v > o ? v : o;
    o = xor_lane_u32<32, true>(v); v = v > o ? v : o;
    return v;
}

// Insert the wave-uniform key x (x != 0, not already present) into a decreasing list;
// the smallest entry falls off the end.
__device__ __forceinline__ u64 insert_desc(u64 list, u64 x)
{
    const u64 up = ((u64)dpp_mov<kDppWaveShr1>((uint32_t)(list >> 32)) << 32) |
                   dpp_mov<kDppWaveShr1>((uint32_t)list);
    const bool keep = list > x;
    const bool prev_keeps = (lane_id() == 0) || (up > x);
    return keep ? list : (prev_keeps ? x : up);
}

// Inclusive prefix sum over the lanes (DPP row shifts, then the row totals are carried over
// with the two row broadcasts).
__device__ __forceinline__ int wave_inclusive_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

}  // namespace dba
