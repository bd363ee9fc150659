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

// ---------------------------------------------------------------------------
// Agent-scope relaxed accesses used for cross-workgroup flags and prefixes.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 load_agent(const u64 *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(u64 *p, u64 v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u32 load_agent(const u32 *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------------------
// Single-pass chained scan across tiles (decoupled look-back). Tile ids are
// handed out by an atomic ticket, so every tile a waiter looks back at has
// already been claimed by a workgroup that is running and that never waits on
// a later tile: every wait ends. As a belt-and-braces measure each wait is
// bounded; a wait that gives up records it in *err and the caller's results
// are then flagged invalid instead of the kernel hanging.
//
// status[t]: bits 63..62 = 0 empty, 1 tile aggregate, 2 inclusive prefix;
// bits 61..0 = value. The array must be zero when the kernel starts.
//
// Must be called by all 64 lanes of ONE wave of the workgroup that owns
// `tile`; returns the exclusive prefix (sum of the aggregates of tiles
// 0..tile-1) in every lane.
// ---------------------------------------------------------------------------
constexpr u64 kFlagAggregate = 1ull << 62;
constexpr u64 kFlagInclusive = 2ull << 62;
constexpr u64 kValueMask = (1ull << 62) - 1ull;
constexpr u32 kSpinLimit = 1u << 22;
constexpr u32 kErrSpin = 1u;

__device__ __forceinline__ u64 lookback_exclusive(u64 *status, u32 tile, u64 aggregate, u32 *err)
{
    const u32 lane = lane_id();
    if (tile == 0) {
        if (lane == 0) store_agent(&status[0], kFlagInclusive | aggregate);
        return 0;
    }
    if (lane == 0) store_agent(&status[tile], kFlagAggregate | aggregate);
    u64 exclusive = 0;
    long long window_end = (long long)tile - 1;
    u32 spins = 0;
    while (true) {
        const long long t = window_end - (long long)lane;
        u64 w = kFlagInclusive;          // lanes that fall before tile 0 contribute nothing
        if (t >= 0) {
            w = load_agent(&status[t]);
            while ((w >> 62) == 0 && spins < kSpinLimit) {
                __builtin_amdgcn_s_sleep(1);
                w = load_agent(&status[t]);
                ++spins;
            }
        }
        const bool gave_up = (w >> 62) == 0;
        if (__any(gave_up)) {
            if (lane == 0) atomicOr(err, kErrSpin);
            break;
        }
        const u64 incl = __ballot((w >> 62) == 2);
        const int first = incl ? (__ffsll((unsigned long long)incl) - 1) : kWave;
        const u64 part = ((int)lane <= first) ? (w & kValueMask) : 0ull;
        exclusive += wave_sum_u64(part);
        if (incl) break;
        window_end -= kWave;
    }
    if (lane == 0) store_agent(&status[tile], kFlagInclusive | ((exclusive + aggregate) & kValueMask));
    return exclusive;
}

// ---------------------------------------------------------------------------
// "Last workgroup out" detector: every workgroup calls it once after its
// global writes; exactly one workgroup (the last to arrive) gets true, and it
// may then read what all the others wrote. `counter` must be zero when the
// kernel starts.
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool last_block_done(u32 *counter, u32 *lds_flag)
{
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const u32 prev = atomicAdd(counter, 1u);
        *lds_flag = (prev == gridDim.x - 1u) ? 1u : 0u;
    }
    __syncthreads();
    const bool last = *lds_flag != 0u;
    if (last) __threadfence();
    return last;
}

__host__ __device__ constexpr u64 align_up(u64 x, u64 a) { return (x + a - 1) / a * a; }

}  // namespace rtopk
