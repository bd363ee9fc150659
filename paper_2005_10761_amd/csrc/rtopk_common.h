// Device-side building blocks shared by the encode and aggregate kernels
// (gfx950, wave64). Nothing here is specific to one kernel.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rtopk {

constexpr int kWave = 64;

using u32 = uint32_t;
using u64 = uint64_t;

// ---------------------------------------------------------------------------
// Sampling key of Definition 3's uniform k-subset: Philox4x32-10 (Salmon et
// al., SC'11) with counter (index, 0, step_lo, step_hi) and key (seed_lo,
// seed_hi); the key is the first two output words, word0 in the high half.
// ---------------------------------------------------------------------------
struct PhiloxSeed {
    u32 seed_lo, seed_hi, step_lo, step_hi;
};

__device__ __forceinline__ u64 sample_key(u32 index, const PhiloxSeed &s)
{
    u32 c0 = index, c1 = 0u, c2 = s.step_lo, c3 = s.step_hi;
    u32 k0 = s.seed_lo, k1 = s.seed_hi;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const u32 hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const u32 hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const u32 n0 = hi1 ^ c1 ^ k0;
        const u32 n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return ((u64)c0 << 32) | (u64)c1;
}

// ---------------------------------------------------------------------------
// Wave-level helpers.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u32 lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ u64 lanes_below() { return (1ull << lane_id()) - 1ull; }

// inclusive prefix sum over the 64 lanes of a wave
__device__ __forceinline__ u32 wave_inclusive_sum(u32 v)
{
    const u32 lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const u32 t = __shfl_up(v, off, kWave);
        if (lane >= (u32)off) v += t;
    }
    return v;
}

__device__ __forceinline__ u64 wave_sum_u64(u64 v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__host__ __device__ constexpr u64 align_up(u64 x, u64 a) { return (x + a - 1) / a * a; }

}  // namespace rtopk
