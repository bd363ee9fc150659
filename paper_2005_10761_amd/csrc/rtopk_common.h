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
        // one 32 x 32 -> 64 bit multiply per product (both halves from one instruction)
        const u64 p0 = (u64)0xD2511F53u * c0, p1 = (u64)0xCD9E8D57u * c2;
        const u32 hi0 = (u32)(p0 >> 32), lo0 = (u32)p0;
        const u32 hi1 = (u32)(p1 >> 32), lo1 = (u32)p1;
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

// Data-parallel-primitive move: every lane reads `v` from the lane the DPP
// control selects inside its row of 16 (or, for the two row broadcasts, from
// the last lane of the previous row / of the first half); lanes the row and
// bank masks leave out, or whose source does not exist, get 0.
template <int kCtrl, int kRowMask, int kBankMask>
__device__ __forceinline__ u32 dpp_or_zero(u32 v)
{
    return (u32)__builtin_amdgcn_update_dpp(0, (int)v, kCtrl, kRowMask, kBankMask, false);
}

// Inclusive prefix sum over the 64 lanes of a wavefront in seven DPP adds
// (a few cycles each; a shuffle goes through the LDS crossbar and costs a
// hundred): a 4-wide window with row_shr 1..3, widened to the row of 16 with
// row_shr 4 and 8 on the upper banks, then the row totals handed on with
// row_bcast 15 (to rows 1 and 3) and row_bcast 31 (to rows 2 and 3).
__device__ __forceinline__ u32 wave_inclusive_sum(u32 v)
{
    u32 x = v;
    x += dpp_or_zero<0x111, 0xF, 0xF>(v);
    x += dpp_or_zero<0x112, 0xF, 0xF>(v);
    x += dpp_or_zero<0x113, 0xF, 0xF>(v);
    x += dpp_or_zero<0x114, 0xF, 0xE>(x);
    x += dpp_or_zero<0x118, 0xF, 0xC>(x);
    x += dpp_or_zero<0x142, 0xA, 0xF>(x);
    x += dpp_or_zero<0x143, 0xC, 0xF>(x);
    return x;
}

// largest value over the wavefront, in every lane: the same seven DPP steps
// with max in place of +, 0 (what a missing source lane reads as) being neutral
__device__ __forceinline__ u32 wave_max_dpp(u32 v)
{
    auto mx = [](u32 a, u32 b) { return a > b ? a : b; };
    u32 x = v;
    x = mx(x, dpp_or_zero<0x111, 0xF, 0xF>(v));
    x = mx(x, dpp_or_zero<0x112, 0xF, 0xF>(v));
    x = mx(x, dpp_or_zero<0x113, 0xF, 0xF>(v));
    x = mx(x, dpp_or_zero<0x114, 0xF, 0xE>(x));
    x = mx(x, dpp_or_zero<0x118, 0xF, 0xC>(x));
    x = mx(x, dpp_or_zero<0x142, 0xA, 0xF>(x));
    x = mx(x, dpp_or_zero<0x143, 0xC, 0xF>(x));
    return (u32)__builtin_amdgcn_readlane((int)x, kWave - 1);
}

// sum over the wavefront, in every lane
__device__ __forceinline__ u32 wave_sum(u32 v)
{
    return (u32)__builtin_amdgcn_readlane((int)wave_inclusive_sum(v), kWave - 1);
}

// smallest / largest value over the wavefront, in every lane (rare paths only:
// six exchanges through the LDS crossbar)
__device__ __forceinline__ u32 wave_min(u32 v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const u32 w = (u32)__shfl_xor((int)v, o, kWave);
        v = w < v ? w : v;
    }
    return v;
}

__device__ __forceinline__ u32 wave_max(u32 v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        const u32 w = (u32)__shfl_xor((int)v, o, kWave);
        v = w > v ? w : v;
    }
    return v;
}

__host__ __device__ constexpr u64 align_up(u64 x, u64 a) { return (x + a - 1) / a * a; }

}  // namespace rtopk
