// Wavefront-level selection primitives for gfx950 (64 lanes).
//
// A "list" is 64 keys, one per lane, sorted in decreasing order; unused places
// hold 0.  Keys are 64-bit and strictly ordered: the high word is an
// order-preserving image of an fp32 score, the low word is the complement of
// the flat coordinate h*V+w, so "greater key" means "higher score, then lower
// coordinate" - the tie rule of the step - and no two live keys are equal.
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
__device__ __forceinline__ float key_score(u64 key) { return float_from_ord((uint32_t)(key >> 32)); }

// Wave-uniform read of one lane's key (lane index must be wave-uniform).
__device__ __forceinline__ u64 read_lane(u64 v, int l)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 umax64(u64 a, u64 b) { return a > b ? a : b; }
__device__ __forceinline__ u64 umin64(u64 a, u64 b) { return a < b ? a : b; }

// Full bitonic sort of one key per lane, decreasing by lane.
__device__ __forceinline__ u64 sort64_desc(u64 key)
{
    const int lane = lane_id();
#pragma unroll
    for (int k2 = 2; k2 <= kWave; k2 <<= 1) {
#pragma unroll
        for (int j = k2 >> 1; j > 0; j >>= 1) {
            const u64 other = __shfl_xor(key, j, kWave);
            const bool desc_block = (lane & k2) == 0;   // k2 == 64: every lane
            const bool lower = (lane & j) == 0;
            key = (lower == desc_block) ? umax64(key, other) : umin64(key, other);
        }
    }
    return key;
}

// a, b: decreasing lists.  Returns the 64 greatest of their union, decreasing.
__device__ __forceinline__ u64 merge_desc(u64 a, u64 b)
{
    const int lane = lane_id();
    const u64 b_rev = __shfl(b, kWave - 1 - lane, kWave);
    u64 c = umax64(a, b_rev);                           // bitonic, holds the top 64
#pragma unroll
    for (int j = kWave >> 1; j > 0; j >>= 1) {
        const u64 other = __shfl_xor(c, j, kWave);
        c = ((lane & j) == 0) ? umax64(c, other) : umin64(c, other);
    }
    return c;
}

// Insert the wave-uniform key x (x != 0, not already present) into a decreasing list;
// the smallest entry falls off the end.
__device__ __forceinline__ u64 insert_desc(u64 list, u64 x)
{
    const int lane = lane_id();
    const u64 up = __shfl_up(list, 1, kWave);
    const bool keep = list > x;
    const bool prev_keeps = (lane == 0) || (up > x);
    return keep ? list : (prev_keeps ? x : up);
}

// Inclusive prefix sum over the lanes.
__device__ __forceinline__ int wave_inclusive_sum(int v)
{
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

}  // namespace dba
