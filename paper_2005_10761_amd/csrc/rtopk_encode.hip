// rtopk_encode: one node-side step of Algorithm 1 (error compensation, the
// rTop-k operator of Definition 3, residual write-back) as a chain of seven
// gfx950 kernels that stream the gradient and the residual exactly once
// (12d bytes). All cross-kernel state lives in the caller's workspace.
//
// The vector is cut into W short contiguous chunks, and every chunk owns a
// slice of the candidate buffer S an eighth as long as the chunk (one byte of
// workspace per element). The wavefront that streams a chunk appends the
// entries it keeps to the chunk's slice in index order and finally stores how
// many it kept. S is therefore ordered by index without any cross-workgroup
// scan, ticket or fence. A chunk that keeps more than its slice holds only
// counts on; the later kernels read such a chunk from the residual buffer,
// which holds a by then. Later kernels walk S chunk by chunk; each of their
// wavefronts takes every U-th chunk, so that a region of the vector that is
// dense in candidates is shared by all wavefronts.
//
// Pipeline:
//   sample     a = g + m at 16384 jittered, stratified locations (4 elements
//              each); clears the control block
//   estimate   one workgroup: from the sample's order statistics, a lower
//              bound t_lo that the r-th largest magnitude exceeds and an upper
//              bound t_hi that it stays below, both with ~6 sigma of margin;
//              [t_lo, t_hi] becomes the finely binned part of the histogram
//   fused      a = g + m, stored into the residual buffer (12d bytes, the
//              dominant kernel); entries with magnitude >= t_lo -> S, and
//              into the workgroup's own histogram row: up to 2048 linear bins
//              over the fine range and one bin for everything above it
//              (every row also carries the sums over groups of 64 bins)
//   pick       one workgroup: the group sums of all rows -> the group that
//              holds the r-th largest magnitude; that group's bins of all
//              rows -> the bin that holds it (the deciding bin)
//   classify   entries of S above the deciding bin are certain members of
//              the top-r set: their Philox key is compared with an a-priori
//              window [K_lo, K_hi] around the k-th smallest of r uniform
//              keys - below: certain winner (counted per chunk), inside:
//              copied to the short list M. Entries inside the deciding bin
//              are copied to the short list B and counted per chunk
//   finalize   one workgroup: exact r-th largest (magnitude, lower index
//              first) inside B -> (T, I*); members of B join the key lists;
//              exact (k - #certain)-th smallest (key, index) in M -> (K*, J*);
//              prefix sum of the winners per chunk. When B overflowed because
//              the deciding bin is one long run of equal magnitudes (zeros,
//              signs, a few levels), the last member is the entry of a known
//              rank in index order and is located from the per-chunk counts.
//              When a short list overflowed otherwise or the key window
//              missed, the same quantities are found by radix selection over
//              all of S instead (exact; on all workgroups of the kernel's
//              grid when the vector is long, see grid_select96)
//   emit       entries of S that are members and winners -> the message in
//              index order, starting at the chunk's prefix; residual at the
//              sent positions <- a - a
// Two special cases of Definition 3 take shortcuts: with k == r (top-k) no
// sampling key is ever computed, and with r == d (random-k) no magnitude is
// ever compared: the streaming kernel then keeps the elements whose key lies
// at or below the upper end of the a-priori window, and sample, estimate,
// and pick are not launched at all.
//
// Every kernel serves up to 16 independent vectors of equal sizes per launch
// (blockIdx.z is the member; rtopk_encode_batch), each with its own slice of
// the workspace and computed exactly as if it were alone.
//
// If the sample misleads the estimate so far that S holds fewer than r
// entries, the histogram shows it; pick then raises a flag and classify,
// finalize and emit walk the vector a itself instead of S (slow, exact).
//
// What the hardware punishes shaped this: a device-scope fence inside a
// kernel costs tens of microseconds once a few hundred workgroups execute
// one, atomics on a single address retire at about one per 12 ns, and
// atomics on one 64-byte line queue behind each other too. So on the ordinary
// path no kernel uses a fence, a ticket or a "last workgroup out" protocol and
// workgroups never wait for each other; histograms are accumulated in LDS and
// stored as plain rows; global atomics only go to per-chunk counters. Only the
// rare exact selection over all candidates lets the workgroups of one grid
// meet at barriers, and those have no device-scope fence (grid_barrier).
#include "rtopk_common.h"
#include "../../include/rtopk.h"
#include "../../include/rtopk_diag.h"

#include <math.h>
#include <cstddef>
#include <mutex>
#include <type_traits>
#include <vector>

namespace rtopk {

constexpr u32 kMaxFineBins = 2048;            // linear bins over [t_lo, fine_hi]: 64 .. 2048, by r
constexpr u32 kCoarseBins = 64;               // one more group of bins, of which only the first is used:
                                              // everything above the linear bins
constexpr u32 kMaxBins = kMaxFineBins + kCoarseBins;
constexpr u32 kMaxFusedBlocks = 256;          // rows of per-workgroup histograms (one per compute unit)
constexpr u32 kCoarseSpan = 64;               // bins per group: every row also carries its group sums
constexpr u32 kMaxGroups = kMaxBins / kCoarseSpan;
static_assert(kMaxBins % kCoarseSpan == 0 && kCoarseSpan == 64, "one lane per bin of a group");

constexpr u32 kSampleLoc = 16384;             // sampled locations, 4 consecutive elements each
constexpr u32 kSampleThreads = 256;
constexpr u32 kEstThreads = 1024;
constexpr u32 kNoSample = 0xFFFFFFFFu;

constexpr u32 kChunkQuantum = 256;            // one wavefront iteration: 64 lanes x 4 elements
constexpr u32 kMinChunk = 4 * kChunkQuantum;  // short vectors: chunks of four iterations
constexpr u32 kTargetChunks = 32768;          // short chunks, dealt round-robin to the wavefronts
constexpr u32 kMaxUnits = 4096;               // wavefronts of classify / emit (per vector)
constexpr u32 kUnitChunks = kTargetChunks / kMaxUnits;   // chunks one of them walks, at most
// In a batch of several vectors the two walking kernels are bound by the
// instructions they issue, a good part of them per wavefront rather than per
// entry: half as many wavefronts then walk twice as many chunks each (eight
// vectors of 25.6 M elements: 23.5 and 20.9 instead of 28 and 23.5 us; one
// vector alone would pay a microsecond in each kernel).
constexpr u32 kBatchUnits = 2048;
constexpr u32 kBatchMembers = 4;              // ... from this many members per launch on
constexpr u32 kUnitChunksMax = kTargetChunks / kBatchUnits;
constexpr u32 kWalkThreads = 256;             // fused / classify / emit workgroups: 4 wavefronts
constexpr u32 kWalkWaves = kWalkThreads / kWave;
constexpr u32 kMaxWalkBlocks = kMaxUnits / kWalkWaves;

// The numbers of candidates kept per chunk are stored unit by unit: the UC
// chunks u, u + U, u + 2U, ... that one walking wavefront takes lie next to
// each other, so it reads them as one 32- or 64-byte piece instead of UC
// separate cache lines.
__host__ __device__ inline u32 chunk_slot(u32 s, u32 U, u32 UC) { return (s % U) * UC + s / U; }
constexpr u32 kListCap = 128;                 // short-list slots per classify workgroup
constexpr u32 kSliceDiv = 8;                  // a chunk's slice of S holds a kSliceDiv-th of the chunk
constexpr int kFinThreads = 1024;
constexpr u32 kFinWaves = kFinThreads / kWave;
constexpr u32 kSlabs = kTargetChunks / (4 * kFinThreads);  // 16-byte groups of chunk counters per thread
constexpr u32 kStageB = 2048, kStageM = 4096; // short lists that fit are selected in LDS (cfg3: 600 and 2,700 entries)

constexpr u32 kErrSelect = 2u;                // a selection found no element of the requested rank
constexpr u32 kErrCount = 4u;                 // the winners did not add up to k
constexpr u32 kErrBarrier = 8u;               // a workgroup gave up waiting for the others of its grid

// The exact fallback over ALL candidates (or over the vector itself) runs on
// kWideBlocks workgroups of the finalize kernel when the vector is long enough
// to be worth it; they exchange 256-bin histograms through the workspace and
// meet at a barrier between radix passes.
constexpr u32 kWideBlocks = 256;              // one per compute unit, shared by the members of a batch
constexpr u32 kWideMinChunks = 256;
constexpr u32 kWidePasses = 24;               // 8 (magnitude, index) + 12 (key, index) + slack; the last two
                                              // `found` slots hold the two selected strings
constexpr u32 kWideSpinLimit = 1u << 20;      // polls (about a microsecond each) before giving up
constexpr u32 kWideCheckInLimit = 1u << 14;   // ... while the workgroups gather for the first time
constexpr u32 kWideGo = 1u, kWideAbort = 2u;

struct WideScratch {
    u32 arrived;                              // workgroups that reached a barrier, over all barriers
    u32 decision;                             // 0, kWideGo (all are resident) or kWideAbort
    u32 pad[62];
    u32 hist[kWidePasses][256];
    u64 found[kWidePasses][2];                // the one string left under a resolved prefix
};

// Histogram geometry chosen by the estimate kernel.
struct Bins {
    u32 t_lo;           // candidates are the entries with magnitude pattern >= t_lo
    u32 fine_hi;        // last pattern of the linear bins
    u32 shift;          // log2 of the patterns per linear bin
    u32 nfine;          // number of linear bins
};

__device__ __forceinline__ u32 bin_of(const Bins &b, u32 m)
{
    return m <= b.fine_hi ? (m - b.t_lo) >> b.shift : b.nfine;
}

__device__ __forceinline__ void bin_range(const Bins &b, u32 bin, u32 *lo, u32 *hi)
{
    if (bin < b.nfine) {
        *lo = b.t_lo + (bin << b.shift);
        const u32 h = *lo + ((1u << b.shift) - 1u);
        *hi = h < b.fine_hi ? h : b.fine_hi;
    } else {
        // the one bin above the linear ones
        *lo = b.fine_hi + 1u;
        *hi = 0x7FFFFFFFu;
    }
}

struct EncodeCtl {
    u32 err;
    u32 path;           // 0: short lists; bit 0: some quantity came from selection over all
                        // candidates; bit 2: the threshold lies in a long run of equal magnitudes
    // written by k_estimate
    Bins bins;
    u32 n_samples;
    // written by k_pick (dense also by k_finalize when r == d and the key window missed)
    u32 dense;          // S holds fewer than r entries: walk the vector itself
    u32 bd_lo, bd_hi;   // pattern range of the deciding bin
    u32 bd_bits;        // bit width of bd_hi - bd_lo
    u64 c_def;          // entries above bd_hi
    // written by k_classify
    u32 overflow;       // a short-list region of some classify workgroup was full
    u32 overflow_m;     // ... and it was a region of the key list M
    // written by k_finalize
    u32 T, I_star;      // last member of the top-r set in (magnitude desc, index asc) order
    u64 K_star;         // last winner in (key asc, index asc) order
    u32 J_star;
    u32 n_b, n_m;
    u32 W, U, UC;       // chunks and their share-out, for the host-side statistics
    u64 count_greater, ties;
};

// (the error word is the first word of the workspace: callers may read it there)
static_assert(offsetof(EncodeCtl, err) == 0, "the error flags lead the control block");

// Geometry and sampling window: a pure function of (d, r, k), computed on the host.
struct Geom {
    u64 d, r, k;
    u32 C;              // elements per chunk (multiple of 256, at least 1024)
    u32 cap;            // entries a chunk's slice of S holds (C / kSliceDiv); a chunk that keeps
                        // more is read from the vector itself by the later kernels
    u32 W;              // chunks
    u32 U;              // wavefronts of classify / emit; wavefront u walks chunks u, u + U, ...
    u32 UC;             // ... at most this many of them (W <= U * UC)
    u32 G3;             // classify / emit workgroups
    u32 L;              // sampled locations
    u32 nfine;          // linear histogram bins
    u32 force_dense;    // diagnostics: make the estimate keep nothing, as if the sample had misled it
    u32 force_abort;    // diagnostics: the workgroups of the wide selection decide "abort" at check-in
    u32 force_timeout;  // diagnostics: the barriers of the wide selection give up at their first poll
    u32 force_low;      // diagnostics: the bracket's upper end is put at its lower end, as if the sample
                        // had underestimated the r-th largest magnitude: it then lies above the linear bins
    u32 take_all;       // k == r: every member is sent, keys are never looked at
    u32 all_members;    // r == d: every coordinate is a member, magnitudes are never looked at
    u32 k_nlz;          // leading zeros of K_hi - K_lo
    u64 K_lo, K_hi;     // key window
};

struct EncodeLayout {
    u64 ctl, wide, zero_bytes, partials, group_sums;
    u64 samples, seg_count, win_cnt, bd_cnt, chunk_base, blk_sure, n_m, n_b, blk_bmin, blk_bmax;
    u64 m_key, m_idx, b_mag, b_idx;
    u64 dm_key, dm_idx, db_key, db_idx;
    u64 s_ent;
    u64 total;
};

static Geom make_geom(u64 d, u64 r, u64 k)
{
    Geom g{};
    g.d = d; g.r = r; g.k = k;
    u64 per = (d + kTargetChunks - 1) / kTargetChunks;
    per = (per + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    if (per < kMinChunk) per = kMinChunk;
    // Measured with a plain streaming add over 66 M and 268 M elements: when every
    // wavefront's piece starts a multiple of 8 KB after its neighbour's (chunks of
    // 2048, 3072, 4096 elements) the stream runs 5-9% slower than with 1024, 2304,
    // 2560 or 8192 elements; a quarter of a kilobyte more staggers the starting points.
    if (per > kMinChunk && per % 1024 == 0 && per % 8192 != 0) per += kChunkQuantum;
    g.C = (u32)per;
    g.cap = g.C / kSliceDiv;
    g.W = (u32)((d + per - 1) / per);
    g.U = g.W < kMaxUnits ? g.W : kMaxUnits;
    g.UC = kUnitChunks;
    g.G3 = (g.U + kWalkWaves - 1) / kWalkWaves;       // (the layout is sized for this many)
    const u64 loc = (d + 3) / 4;
    g.L = (u32)(loc < kSampleLoc ? loc : kSampleLoc);
    // Every workgroup of the streaming kernel stores its whole histogram: few
    // bins when r is small (the list B of the deciding bin then holds a few
    // hundred entries anyway), more when r is large.
    g.nfine = 256;
    while (g.nfine < kMaxFineBins && (u64)g.nfine * 256 < r) g.nfine *= 2;
    g.take_all = (k == r) ? 1u : 0u;
    g.all_members = (r == d) ? 1u : 0u;
    // The number of members with key below x * 2^64 is Binomial(r, x). The
    // window keeps 7 standard deviations plus a constant (for small k, where
    // the normal approximation is poor) on both sides of k; a miss is still
    // resolved exactly, only slowly.
    const long double two64 = 18446744073709551616.0L;
    const long double kk = (long double)k, rr = (long double)r;
    const long double slack = 7.0L * sqrtl(kk * (1.0L - kk / rr)) + 30.0L;
    const long double lo = (kk - slack) / rr, hi = (kk + slack) / rr;
    g.K_lo = lo <= 0.0L ? 0ull : (u64)(lo * two64);
    g.K_hi = hi >= 1.0L ? ~0ull : (u64)(hi * two64);
    if (g.K_hi < g.K_lo) g.K_hi = g.K_lo;
    const u64 width = g.K_hi - g.K_lo;
    g.k_nlz = width ? (u32)__builtin_clzll(width) : 63u;
    return g;
}

// the walking kernels' share-out for a launch that serves nb vectors (see kBatchUnits)
static void set_units(Geom &g, unsigned nb)
{
    const u32 units = nb >= kBatchMembers ? kBatchUnits : kMaxUnits;
    g.U = g.W < units ? g.W : units;
    g.UC = nb >= kBatchMembers ? kUnitChunksMax : kUnitChunks;
    g.G3 = (g.U + kWalkWaves - 1) / kWalkWaves;
}

static EncodeLayout make_layout(const Geom &g)
{
    EncodeLayout L{};
    u64 o = 0;
    auto take = [&](u64 bytes) { u64 at = o; o = align_up(o + bytes, 256); return at; };
    L.ctl = take(sizeof(EncodeCtl));
    L.wide = take(sizeof(WideScratch));
    L.zero_bytes = o;                       // cleared at the start of every call
    L.partials = take((u64)kMaxFusedBlocks * kMaxBins * 4);
    L.group_sums = take((u64)kMaxFusedBlocks * kMaxGroups * 4);
    L.samples = take((u64)kSampleLoc * 16);
    L.seg_count = take((u64)kTargetChunks * 4);      // fixed size: its offset depends on nothing
    L.win_cnt = take((u64)kTargetChunks * 4);
    L.bd_cnt = take((u64)kTargetChunks * 4);
    L.chunk_base = take((u64)kTargetChunks * 4);
    L.blk_sure = take((u64)g.G3 * 4);
    L.n_m = take((u64)g.G3 * 4);
    L.n_b = take((u64)g.G3 * 4);
    L.blk_bmin = take((u64)g.G3 * 4);
    L.blk_bmax = take((u64)g.G3 * 4);
    const u64 slots = (u64)g.G3 * kListCap;
    L.m_key = take(slots * 8);
    L.m_idx = take(slots * 4);
    L.b_mag = take(slots * 4);
    L.b_idx = take(slots * 4);
    L.dm_key = take(2 * slots * 8);
    L.dm_idx = take(2 * slots * 4);
    L.db_key = take(slots * 8);
    L.db_idx = take(slots * 4);
    L.s_ent = take((u64)g.W * g.cap * 8);
    L.total = o;
    return L;
}

__device__ __forceinline__ u32 mag_of(u32 bits) { return bits & 0x7FFFFFFFu; }
__device__ __forceinline__ u32 popc64(u64 m) { return (u32)__popcll((unsigned long long)m); }

// Workgroup barrier that orders LDS accesses only: global loads, stores and
// atomics a thread has in flight stay in flight (__syncthreads would wait for
// all of them to complete first).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Orders one wavefront's own LDS accesses: what its lanes wrote before is what
// its lanes read after (the hardware keeps a wavefront's LDS operations in
// order; this keeps the compiler from moving them).
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// ---------------------------------------------------------------------------
// workgroup-wide sums of one value per thread (thread order); the second
// level is a wavefront scan, not a serial loop: LDS round trips are slow
// ---------------------------------------------------------------------------
// exclusive prefix of v over the workgroup; the grand total is left in lds[waves]
__device__ __forceinline__ u32 block_exclusive_sum(u32 v, u32 *lds /* >= waves + 1 words */)
{
    const u32 lane = lane_id(), wave = threadIdx.x / kWave, nw = blockDim.x / kWave;
    const u32 inc = wave_inclusive_sum(v);
    if (lane == kWave - 1) lds[wave] = inc;
    lds_barrier();
    if (wave == 0) {
        const u32 x = lane < nw ? lds[lane] : 0u;
        const u32 xi = wave_inclusive_sum(x);
        if (lane < nw) lds[lane] = xi - x;
        if (lane == nw - 1) lds[nw] = xi;
    }
    lds_barrier();
    const u32 res = lds[wave] + inc - v;
    lds_barrier();
    return res;
}

// sum of v over the workgroup, in every thread (the sum must fit 32 bits)
__device__ __forceinline__ u32 block_sum(u32 v, u32 *lds /* >= waves words */)
{
    const u32 nw = blockDim.x / kWave;
    v = wave_sum(v);
    if (lane_id() == 0) lds[threadIdx.x / kWave] = v;
    lds_barrier();
    const u32 total = wave_sum(lane_id() < nw ? lds[lane_id()] : 0u);
    lds_barrier();
    return total;
}

// ---------------------------------------------------------------------------
// sample: magnitudes of a = g + m at g.L locations, one per stratum of the
// vector, at a hashed offset inside the stratum, four consecutive elements
// each. Also clears what later kernels accumulate into.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 stratum_start(const Geom &g, u32 j)
{
    // strata of (almost) equal length; only monotonicity and the two ends matter
    if (j >= g.L) return g.d;
    static_assert((kSampleLoc & (kSampleLoc - 1)) == 0, "the usual count of strata is a power of two");
    const u64 x = g.L == kSampleLoc ? (g.d * (u64)j) / kSampleLoc     // d * j < 2^46; a shift
                                    : (u64)((double)g.d * (double)j / (double)g.L);
    return x < g.d ? x : g.d;
}

__device__ __forceinline__ void
sample_body(const float *__restrict__ grad, const float *__restrict__ residual, Geom g,
         PhiloxSeed seed, u32 *__restrict__ zero_base, u32 zero_words, u32 *__restrict__ samples)
{
    const u32 j = blockIdx.x * kSampleThreads + threadIdx.x;
    for (u32 i = j; i < zero_words; i += gridDim.x * kSampleThreads) zero_base[i] = 0u;
    if (j >= kSampleLoc) return;
    u32 out[4] = {kNoSample, kNoSample, kNoSample, kNoSample};
    if (j < g.L) {
        const u64 start = stratum_start(g, j), end = stratum_start(g, j + 1);
        const u64 len = end - start;
        u64 p = start;
        if (len > 4) {
            // The offset depends on the stratum AND on (seed, step): a vector whose
            // layout happens to mislead one set of offsets (a period close to the
            // stratum length) does not mislead the next step's or another worker's.
            // Which elements are sampled never changes the result, only the path.
            u32 hsh = (j + 1u) * 0x9E3779B1u;
            hsh ^= seed.seed_lo * 0x85EBCA77u + seed.step_lo * 0xC2B2AE3Du +
                   (seed.seed_hi ^ seed.step_hi) * 0x27D4EB2Fu;
            hsh ^= hsh >> 15; hsh *= 0x85EBCA77u; hsh ^= hsh >> 13;
            hsh *= 0xC2B2AE3Du; hsh ^= hsh >> 16;
            // offset in [0, len - 4], scaled from the hash instead of a remainder
            p += (u64)(((u64)hsh * (u64)(len - 3)) >> 32);
        }
        const bool aligned = (((uintptr_t)grad | (uintptr_t)residual) & 15u) == 0;
        if (aligned && len > 4 && (p & ~3ull) + 4 <= g.d) {
            // one 16-byte load per array, from one cache line each (the four elements
            // may start up to three before the stratum: it stays a spread-out sample)
            p &= ~3ull;
            const float4 gv = *reinterpret_cast<const float4 *>(grad + p);
            const float4 mv = *reinterpret_cast<const float4 *>(residual + p);
            out[0] = mag_of(__float_as_uint(gv.x + mv.x));
            out[1] = mag_of(__float_as_uint(gv.y + mv.y));
            out[2] = mag_of(__float_as_uint(gv.z + mv.z));
            out[3] = mag_of(__float_as_uint(gv.w + mv.w));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const u64 i = p + e;
                if (i < end) out[e] = mag_of(__float_as_uint(grad[i] + residual[i]));
            }
        }
    }
    reinterpret_cast<uint4 *>(samples)[j] = make_uint4(out[0], out[1], out[2], out[3]);
}

// ---------------------------------------------------------------------------
// estimate: order statistics of the sample -> histogram geometry.
// With n samples and p = r/d, the number of samples among the true top r is
// about Binomial(n, p); clusters of four that rise and fall together double
// the standard deviation at worst. t_lo is the lower edge of the 12-bit
// pattern bucket that holds the sample of rank np + 6 sd + 8 (so that at
// least r entries lie at or above t_lo), t_hi the upper edge of the bucket
// that holds the sample of rank np - 6 sd - 8 (fewer than r entries lie
// above it).
// ---------------------------------------------------------------------------
// One wavefront: walking 4096 buckets (in LDS) downwards from the bucket
// `top` (nothing lies above it), 256 buckets at a time, find for each of
// NRANKS ranks the bucket b with #(buckets above b) < need <= #(buckets >= b).
// Stores b and the population above it; stores nothing for a rank that all
// buckets together do not reach. The samples that matter sit in the few
// buckets under the largest one: one or two steps instead of a walk over all.
template <int NRANKS>
__device__ __forceinline__ void wave_pick_from_top(const u32 *hist, u32 top, const u32 (&need)[NRANKS],
                                                   u32 *out_bin, u32 *out_before)
{
    const u32 lane = lane_id();
    u32 above = 0;
    bool pending[NRANKS];
#pragma unroll
    for (int k = 0; k < NRANKS; ++k) pending[k] = true;
    for (int hi = (int)(top | 255u); hi >= 0; hi -= 256) {
        u32 c[4];
        u32 mine = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) { c[q] = hist[hi - 4 * (int)lane - q]; mine += c[q]; }
        const u32 inc = wave_inclusive_sum(mine);
        const u32 before = above + inc - mine;
        bool any = false;
#pragma unroll
        for (int k = 0; k < NRANKS; ++k) {
            const bool here = pending[k] && before < need[k] && need[k] <= before + mine;
            if (here) {
                u32 run = before;
                bool done = false;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (!done && run + c[q] >= need[k]) {
                        out_bin[k] = (u32)(hi - 4 * (int)lane - q);
                        out_before[k] = run;
                        done = true;
                    }
                    run += c[q];
                }
            }
            if (__ballot(here) != 0ull) pending[k] = false;
            any = any || pending[k];
        }
        if (!any) break;
        above += (u32)__builtin_amdgcn_readlane((int)inc, kWave - 1);
    }
}

__device__ __forceinline__ void
estimate_body(const u32 *__restrict__ samples, Geom g, EncodeCtl *ctl)
{
    // One compute unit looks at 65,536 samples: the work per sample is what this
    // kernel costs, so the two passes over them are a handful of instructions per
    // 16-byte group. A sample is a magnitude pattern (< 2^31) or kNoSample
    // (all ones): as signed integers the missing ones are -1, below every real one.
    __shared__ u32 h_max[4096];                           // buckets of the per-thread maxima
    __shared__ u32 h[4096];                               // buckets of the samples that matter
    __shared__ u32 scan_lds[kEstThreads / kWave + 1];
    __shared__ u32 bin_s[3], before_s[3], top_s;
    const u32 tid = threadIdx.x;
    constexpr u32 kVecs = kSampleLoc / kEstThreads;       // 16-byte sample groups per thread
    const uint4 *s4 = reinterpret_cast<const uint4 *>(samples);
    uint4 v[kVecs];
#pragma unroll
    for (u32 q = 0; q < kVecs; ++q) v[q] = s4[q * kEstThreads + tid];
    for (u32 b = tid; b < 4096u; b += kEstThreads) { h[b] = 0u; h_max[b] = 0u; }
    if (tid < 3u) { bin_s[tid] = 0u; before_s[tid] = 0u; }
    if (tid == 0) top_s = 0u;
    auto smax = [](int a, int b) { return a > b ? a : b; };
    int gmax[kVecs];                                      // largest of each group, -1 if none
    int tmax = -1;
#pragma unroll
    for (u32 q = 0; q < kVecs; ++q) {
        gmax[q] = smax(smax((int)v[q].x, (int)v[q].y), smax((int)v[q].z, (int)v[q].w));
        tmax = smax(tmax, gmax[q]);
    }
    // Number of samples: four per location once every stratum is longer than
    // four elements; counted otherwise (short vectors).
    u32 n;
    if ((u64)g.L * 5ull <= g.d) {
        n = 4u * g.L;
        lds_barrier();                                    // orders the clearing of the histograms
    } else {
        u32 nvalid = 0;
#pragma unroll
        for (u32 q = 0; q < kVecs; ++q)
            nvalid += (v[q].x != kNoSample) + (v[q].y != kNoSample) + (v[q].z != kNoSample) +
                      (v[q].w != kNoSample);
        n = block_sum(nvalid, scan_lds);
    }

    const float p = (float)((double)g.r / (double)g.d);
    const float np = (float)n * p;
    const float sd = 2.0f * sqrtf(np * (1.0f - p));
    const float lo_rank = ceilf(np + 6.0f * sd + 8.0f), hi_rank = floorf(np - 6.0f * sd - 8.0f);
    const bool lo_all = lo_rank > (float)n;       // too few samples below the top: keep everything
    const u32 s_lo = lo_all ? n : (u32)lo_rank;
    const u32 s_hi = hi_rank < 1.0f ? 1u : (u32)hi_rank;

    // Only the top s_lo samples matter. At most s_lo - 1 threads hold a sample
    // above the s_lo-th largest one, so the s_lo-th largest of the per-thread
    // maxima is not above it: buckets below that maximum's bucket need no count.
    // (the bucket of the largest sample of all is where every walk starts)
    {
        const u32 wmax = wave_max_dpp(tmax >= 0 ? (u32)tmax >> 19 : 0u);
        if (lane_id() == 0 && wmax) atomicMax(&top_s, wmax);
    }
    u32 cut_bucket = 0;
    if (s_lo < kEstThreads) {
        if (tmax >= 0) atomicAdd(&h_max[(u32)tmax >> 19], 1u);
        lds_barrier();
        if (tid < kWave) {
            const u32 want_cut[1] = {s_lo};
            wave_pick_from_top<1>(h_max, top_s, want_cut, &bin_s[2], &before_s[2]);
        }
        lds_barrier();
        cut_bucket = bin_s[2];                     // stays 0 when fewer than s_lo threads hold samples
    }
    const int cut = (int)(cut_bucket << 19);       // >= 0: missing samples never pass
    u32 nzero = 0;
    auto count = [&](u32 m) {
        if ((int)m < cut) return;
        if (m == 0u) ++nzero;                     // exact zeros come in long runs: count them aside
        else atomicAdd(&h[m >> 19], 1u);
    };
#pragma unroll
    for (u32 q = 0; q < kVecs; ++q) {
        if (gmax[q] < cut) continue;               // nearly every group
        count(v[q].x); count(v[q].y); count(v[q].z); count(v[q].w);
    }
    nzero = wave_sum(nzero);
    if (lane_id() == 0 && nzero) atomicAdd(&h[0], nzero);
    __syncthreads();
    if (tid < kWave) {
        const u32 want[2] = {s_lo, s_hi};
        wave_pick_from_top<2>(h, top_s, want, &bin_s[0], &before_s[0]);
    }
    __syncthreads();
    if (tid == 0) {
        u32 t_lo = lo_all ? 0u : (bin_s[0] << 19);
        u32 t_hi = (bin_s[1] << 19) | 0x7FFFFu;
        if (g.force_dense) t_lo = 0x7FFFFFFFu;
        if (g.force_low) t_hi = t_lo;
        if (t_hi < t_lo) t_hi = t_lo;
        u32 shift = 0;
        while (((t_hi - t_lo) >> shift) >= g.nfine) ++shift;
        const u64 top = (u64)t_lo + ((u64)g.nfine << shift) - 1ull;
        ctl->bins.t_lo = t_lo;
        ctl->bins.fine_hi = top > 0x7FFFFFFFull ? 0x7FFFFFFFu : (u32)top;
        ctl->bins.shift = shift;
        ctl->bins.nfine = g.nfine;
        ctl->n_samples = n;
    }
}

// ---------------------------------------------------------------------------
// One wavefront iteration of the streaming kernel covers 256 consecutive
// elements starting at `base`. Layout of the four elements a lane holds:
// kVec4 -> base + 4*lane + e (16-byte accesses); otherwise base + 64*e + lane
// (coalesced 4-byte accesses, any alignment). Kept entries are appended to
// the chunk's slice of S in index order.
// ---------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool kVec4>
__device__ __forceinline__ u64 elem_index(u64 base, int e)
{
    return kVec4 ? base + 4ull * lane_id() + (u64)e : base + 64ull * (u64)e + lane_id();
}

template <bool kVec4>
__device__ __forceinline__ void append_hits(const u32 (&bits)[4], const bool (&hit)[4], u64 base,
                                            u32 &run, uint2 *__restrict__ my_ent, u32 cap)
{
    const u64 b0 = __ballot(hit[0]), b1 = __ballot(hit[1]), b2 = __ballot(hit[2]),
              b3 = __ballot(hit[3]);
    if ((b0 | b1 | b2 | b3) == 0ull) return;
    if (run >= cap) {
        // the slice is full: the chunk will be read from the vector itself, only its
        // count goes on (anything above cap says so)
        run += popc64(b0) + popc64(b1) + popc64(b2) + popc64(b3);
        return;
    }
    const u64 below = lanes_below();
    u32 pos[4];
    if (kVec4) {
        u32 p = run + popc64(b0 & below) + popc64(b1 & below) + popc64(b2 & below) +
                popc64(b3 & below);
#pragma unroll
        for (int e = 0; e < 4; ++e) { pos[e] = p; p += hit[e] ? 1u : 0u; }
    } else {
        pos[0] = run + popc64(b0 & below);
        pos[1] = run + popc64(b0) + popc64(b1 & below);
        pos[2] = run + popc64(b0) + popc64(b1) + popc64(b2 & below);
        pos[3] = run + popc64(b0) + popc64(b1) + popc64(b2) + popc64(b3 & below);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (hit[e] && pos[e] < cap) {
            my_ent[pos[e]] = make_uint2((u32)elem_index<kVec4>(base, e), bits[e]);
        }
    }
    run += popc64(b0) + popc64(b1) + popc64(b2) + popc64(b3);
}

// ---------------------------------------------------------------------------
// fused: a = g + m -> residual buffer; candidates -> S and the histogram.
// Reads g and m once, writes a once: 12d bytes of HBM traffic. The grid is
// sized to what the device holds at once; wavefront v takes chunks v,
// v + #wavefronts, ... so that neighbouring wavefronts stream neighbouring
// 4 KB pieces of each array.
// ---------------------------------------------------------------------------
constexpr u32 kFusedThreads = 512;
constexpr u32 kFusedWaves = kFusedThreads / kWave;
// Rows of 256 elements a wavefront fetches together (two 16-byte loads per lane
// and row in flight) before it adds, stores and looks at them. Measured over
// the batched launches of 11 M, 25.6 M and 66 M elements: one row 203 / 445 /
// 591 us, two 173 / 393 / 531, three 178 / 394 / 559, four 174 / 408 / 566.
constexpr int kFusedRows = 2;

// kAll (r == d, the random-k operator): no magnitude decides anything. An
// element is kept when its sampling key lies at or below the upper end of the
// a-priori window (all of them when k == r as well); no histogram is made and
// the control block, which no earlier kernel has touched, is cleared here.
template <bool kVec4, bool kAll>
__device__ __forceinline__ void
fused_body(const float *__restrict__ grad, float *__restrict__ residual, Geom g, PhiloxSeed seed,
        EncodeCtl *__restrict__ ctl, u32 zero_words, u32 *__restrict__ partials,
        u32 *__restrict__ group_sums, u32 *__restrict__ seg_count, uint2 *__restrict__ s_ent)
{
    __shared__ u32 h[kAll ? 1 : kMaxBins];
    Bins bins{};
    u32 nbins = 0;
    if (kAll) {
        // (the control block and what follows it up to zero_words, at the workspace's start)
        if (blockIdx.x == 0)
            for (u32 i = threadIdx.x; i < zero_words; i += kFusedThreads)
                reinterpret_cast<u32 *>(ctl)[i] = 0u;
    } else {
        bins = ctl->bins;
        nbins = bins.nfine + kCoarseBins;
        for (u32 b = threadIdx.x; b < nbins; b += kFusedThreads) h[b] = 0u;
        __syncthreads();
    }

    const u32 wave_stride = gridDim.x * kFusedWaves;
    u32 n_above = 0;        // this wavefront's candidates above the linear bins
    for (u32 w = blockIdx.x * kFusedWaves + threadIdx.x / kWave; w < g.W; w += wave_stride) {
        const u64 c0 = (u64)w * g.C;
        const u64 c1 = c0 + g.C < g.d ? c0 + g.C : g.d;
        uint2 *my_ent = s_ent + (u64)w * g.cap;
        u32 run = 0;
        auto keep = [&](const u32 (&bits)[4], const bool (&valid)[4], u64 base) {
            bool hit[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (kAll) {
                    hit[e] = valid[e] &&
                             (g.take_all != 0u ||
                              sample_key((u32)elem_index<kVec4>(base, e), seed) <= g.K_hi);
                } else {
                    const u32 m = mag_of(bits[e]);
                    hit[e] = valid[e] && m >= bins.t_lo;
                    // candidates inside the bracket are counted bin by bin; the ones above it
                    // (certain members, often most of the candidates and crowded in a few
                    // exponents) only need their number: a popcount instead of LDS additions
                    const bool fine = hit[e] && m <= bins.fine_hi;
                    if (fine) atomicAdd(&h[(m - bins.t_lo) >> bins.shift], 1u);
                    n_above += popc64(__ballot(hit[e] && !fine));
                }
            }
            append_hits<kVec4>(bits, hit, base, run, my_ent, g.cap);
        };
        const bool all_valid[4] = {true, true, true, true};
        // NR full rows at a time, all loads issued before the first use. Every
        // element is read once and written once: both the loads and the store carry
        // the streaming hint. (Measured: the hint on the residual's load AND store
        // together shortens the kernel by 15%; either one alone changes nothing.)
        auto full_rows = [&](auto nr_c, u64 base) {
            constexpr int NR = decltype(nr_c)::value;
            u32 bits[NR][4];
            if (kVec4) {
                const f32x4 *g4 = reinterpret_cast<const f32x4 *>(grad + base) + lane_id();
                f32x4 *m4 = reinterpret_cast<f32x4 *>(residual + base) + lane_id();
                f32x4 gv[NR], mv[NR];
#pragma unroll
                for (int u = 0; u < NR; ++u) {
                    gv[u] = __builtin_nontemporal_load(g4 + u * kWave);
                    mv[u] = __builtin_nontemporal_load(m4 + u * kWave);
                }
#pragma unroll
                for (int u = 0; u < NR; ++u) {
                    const f32x4 a = gv[u] + mv[u];
                    __builtin_nontemporal_store(a, m4 + u * kWave);
                    bits[u][0] = __float_as_uint(a.x); bits[u][1] = __float_as_uint(a.y);
                    bits[u][2] = __float_as_uint(a.z); bits[u][3] = __float_as_uint(a.w);
                }
            } else {
                const float *gp = grad + base + lane_id();
                float *mp = residual + base + lane_id();
                float gv[4 * NR], mv[4 * NR];
#pragma unroll
                for (int q = 0; q < 4 * NR; ++q) {
                    gv[q] = __builtin_nontemporal_load(gp + q * kWave);
                    mv[q] = __builtin_nontemporal_load(mp + q * kWave);
                }
#pragma unroll
                for (int q = 0; q < 4 * NR; ++q) {
                    const float a = gv[q] + mv[q];
                    __builtin_nontemporal_store(a, mp + q * kWave);
                    bits[q / 4][q % 4] = __float_as_uint(a);
                }
            }
#pragma unroll
            for (int u = 0; u < NR; ++u) keep(bits[u], all_valid, base + u * kChunkQuantum);
        };
        u64 base = c0;
        for (; base + kFusedRows * kChunkQuantum <= c1; base += kFusedRows * kChunkQuantum)
            full_rows(std::integral_constant<int, kFusedRows>{}, base);
        for (; base + kChunkQuantum <= c1; base += kChunkQuantum)
            full_rows(std::integral_constant<int, 1>{}, base);
        if (base < c1) {
            u32 bits[4];
            bool valid[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const u64 i = elem_index<kVec4>(base, e);
                valid[e] = i < c1;
                bits[e] = 0u;
                if (valid[e]) {
                    const float a = grad[i] + residual[i];
                    residual[i] = a;
                    bits[e] = __float_as_uint(a);
                }
            }
            keep(bits, valid, base);
        }
        if (lane_id() == 0) seg_count[chunk_slot(w, g.U, g.UC)] = run;
    }
    if (kAll) return;
    if (lane_id() == 0 && n_above != 0u) atomicAdd(&h[bins.nfine], n_above);
    __syncthreads();
    // The workgroup's histogram goes out as one dense row with plain stores:
    // device-wide atomics here, however few, slow the whole stream down. With
    // it go the sums over groups of kCoarseSpan bins: the pick kernel first adds
    // up those (a sixty-fourth of the data), finds the group that holds the
    // r-th largest magnitude and then only needs that group's bins of every row.
    u32 *row = partials + (u64)blockIdx.x * nbins;
    for (u32 b = threadIdx.x; b < nbins; b += kFusedThreads) row[b] = h[b];
    const u32 ngroups = (nbins + kCoarseSpan - 1) / kCoarseSpan;
    for (u32 c = threadIdx.x / kWave; c < ngroups; c += kFusedWaves) {
        const u32 b = c * kCoarseSpan + lane_id();
        const u32 sum = wave_sum(b < nbins ? h[b] : 0u);
        if (lane_id() == 0) group_sums[(u64)blockIdx.x * kMaxGroups + c] = sum;
    }
}

// ---------------------------------------------------------------------------
// The candidates as later kernels see them: chunk s holds count(s) entries
// (index, binary32 pattern), in index order. Normally that is the slice of S
// the fused kernel filled; in dense mode it is the chunk of a itself.
// ---------------------------------------------------------------------------
struct Candidates {
    const u32 *__restrict__ seg_count;
    const uint2 *__restrict__ s_ent;
    const float *__restrict__ a;
    u64 d;
    u32 C, U, UC, cap;
    bool dense;         // every chunk is read from the vector (the estimate kept too little)

    __device__ __forceinline__ u32 length(u32 s) const
    {
        const u64 c0 = (u64)s * C;
        return (u32)(c0 + C < d ? C : d - c0);
    }
    // entries of chunk s, and whether they are the chunk's elements themselves:
    // a chunk that kept more than its slice holds is read from the vector (all
    // its elements then count as entries; what lies below the candidates'
    // lower bound is below every threshold the later kernels compare with)
    __device__ __forceinline__ u32 count(u32 s, bool *from_vector) const
    {
        const u32 kept = dense ? 0u : seg_count[chunk_slot(s, U, UC)];
        *from_vector = dense || kept > cap;
        return *from_vector ? length(s) : kept;
    }
    __device__ __forceinline__ void entry(u32 s, u32 j, bool from_vector, u32 *idx, u32 *bits) const
    {
        if (!from_vector) {
            const uint2 e = s_ent[(u64)s * cap + j];
            *idx = e.x;
            *bits = e.y;
        } else {
            const u64 at = (u64)s * C + j;
            *idx = (u32)at;
            *bits = __float_as_uint(a[at]);
        }
    }
};

// One wavefront walks chunks u, u + U, u + 2U, ... as one flat sequence: lane
// i first fetches the size of the i-th of them (there are at most
// kUnitChunks), a prefix sum turns flat positions into (chunk, entry) pairs,
// and every iteration of the walk hands 64 consecutive positions to the 64
// lanes; the entries of one chunk stay in index order. f(valid, i, index,
// pattern, first, p0) is called by all lanes in every iteration, so it may use
// wave-wide operations; (index, pattern) is the lane's entry, i the ordinal of
// its chunk among the wavefront's chunks, first the flat position of the
// chunk's first entry and p0 the flat position lane 0 holds.
// The same walk serves the slow exact paths of the finalize kernel, where a
// wavefront takes kWave consecutive chunks at a time (kChunks = kWave,
// stride 1).
template <u32 kChunks>
struct ChunkWalk {
    u32 u, stride, excl, inc, total;
    u64 from_vector;        // bit i: the i-th chunk is read from the vector itself
    static constexpr u32 kRowQueueSize = 512; // a power of two >= 63 entries waiting + one row of 256

    // chunks first, first + step, ..., at most kChunks of them and only those below n_chunks
    __device__ __forceinline__ ChunkWalk(const Candidates &cand, u32 first, u32 step, u32 n_chunks)
    {
        static_assert(kChunks <= kWave && (kChunks & (kChunks - 1)) == 0, "one lane per chunk");
        const u32 lane = lane_id();
        u = first;
        stride = step;
        const u64 s = (u64)first + (u64)lane * step;
        bool fv = false;
        u32 cnt = (lane < kChunks && s < n_chunks) ? cand.count((u32)s, &fv) : 0u;
        from_vector = __ballot(fv);
        if (fv) cnt = 0u;           // not part of the flat sequence: see for_each_vector_row
        inc = wave_inclusive_sum(cnt);
        excl = inc - cnt;
        total = __shfl(inc, kWave - 1, kWave);
    }

    // flat position p -> ordinal of its chunk and the flat position of that chunk's first entry
    __device__ __forceinline__ void locate(u32 p, u32 *ordinal, u32 *first) const
    {
        // number of chunks that end at or before position p = ordinal of p's chunk
        u32 c = 0;
#pragma unroll
        for (u32 step = kChunks / 2; step > 0; step >>= 1) {
            const u32 end_of = __shfl(inc, c + step - 1, kWave);
            if (end_of <= p) c += step;
        }
        c &= kChunks - 1;
        *ordinal = c;
        *first = __shfl(excl, c, kWave);
    }

    // f(valid, i, index, pattern, first, p0), see above; the entries of four
    // iterations are fetched together while that many are left
    template <class F>
    __device__ __forceinline__ void for_each(const Candidates &cand, F &&f) const
    {
        const u32 lane = lane_id();
        constexpr u32 kAhead = 4;
        u32 p0 = 0;
        for (; p0 + kAhead * kWave <= total; p0 += kAhead * kWave) {
            u32 c[kAhead], first[kAhead], idx[kAhead], bits[kAhead];
#pragma unroll
            for (u32 q = 0; q < kAhead; ++q) {
                const u32 p = p0 + q * kWave + lane;
                locate(p, &c[q], &first[q]);
                cand.entry(u + c[q] * stride, p - first[q], false, &idx[q], &bits[q]);
            }
#pragma unroll
            for (u32 q = 0; q < kAhead; ++q) f(true, c[q], idx[q], bits[q], first[q], p0 + q * kWave);
        }
        for (; p0 < total; p0 += kWave) {
            const u32 p = p0 + lane;
            u32 c, first, idx = 0, bits = 0;
            locate(p, &c, &first);
            if (p < total) cand.entry(u + c * stride, p - first, false, &idx, &bits);
            f(p < total, c, idx, bits, first, p0);
        }
    }

    // Cursor over the rows of 256 elements of the wavefront's chunks that are read
    // from the vector itself (they kept more candidates than their slice of S
    // holds, or the whole vector is walked): lane l of a row holds the four
    // elements idx0 .. idx0 + 3, idx0 = row start + 4 l, loaded with one 16-byte
    // access where the vector's alignment allows.
    struct RowCursor {
        u64 rest;           // chunks still to come
        u64 c0;             // first element of the current chunk
        u32 i, len, r0;     // its ordinal among the wavefront's chunks, its length, the next row
        bool open;
    };
    __device__ __forceinline__ RowCursor rows() const { return RowCursor{from_vector, 0ull, 0u, 0u, 0u, false}; }
    // moves to the next chunk if the current one is used up; false when no chunk is left
    __device__ __forceinline__ bool next_chunk(const Candidates &cand, RowCursor &rc) const
    {
        if (rc.rest == 0ull) return false;
        rc.i = (u32)__ffsll((unsigned long long)rc.rest) - 1u;
        rc.rest &= rc.rest - 1ull;
        const u32 s = u + rc.i * stride;
        rc.c0 = (u64)s * cand.C;
        rc.len = cand.length(s);
        rc.r0 = 0;
        rc.open = true;
        return true;
    }
    // loads the current chunk's next row (the chunk must have one left)
    __device__ __forceinline__ void load_row(const Candidates &cand, RowCursor &rc, u32 *idx0,
                                             u32 (&bits)[4], bool (&valid)[4]) const
    {
        const u32 off = rc.r0 + 4u * lane_id();
        const bool vec16 = (reinterpret_cast<uintptr_t>(cand.a) & 15u) == 0;
        if (vec16 && rc.r0 + kChunkQuantum <= rc.len) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(cand.a + rc.c0 + off);
            bits[0] = __float_as_uint(v.x); bits[1] = __float_as_uint(v.y);
            bits[2] = __float_as_uint(v.z); bits[3] = __float_as_uint(v.w);
#pragma unroll
            for (u32 e = 0; e < 4; ++e) valid[e] = true;
        } else {
#pragma unroll
            for (u32 e = 0; e < 4; ++e) {
                valid[e] = off + e < rc.len;
                bits[e] = valid[e] ? __float_as_uint(cand.a[rc.c0 + off + e]) : 0u;
            }
        }
        *idx0 = (u32)rc.c0 + off;
        rc.r0 += kChunkQuantum;
        if (rc.r0 >= rc.len) rc.open = false;
    }

    // g(i, idx0, patterns, valid) for every such row, all lanes together, rows of one
    // chunk in index order (rare paths: one row in flight)
    template <class G>
    __device__ __forceinline__ void for_each_vector_row(const Candidates &cand, G &&g) const
    {
        RowCursor rc = rows();
        for (;;) {
            if (!rc.open && !next_chunk(cand, rc)) break;
            u32 idx0, bits[4];
            bool valid[4];
            load_row(cand, rc, &idx0, bits, valid);
            g(rc.i, idx0, bits, valid);
        }
    }

    // The same chunks with the elements that keep(pattern) lets through gathered
    // first, so that the work per entry (a sampling key costs a hundred
    // instructions) is done on full wavefronts: a row's survivors are appended in
    // index order to a ring in LDS (buf: kRowQueue entries owned by this
    // wavefront) and taken from its front 64 at a time; what is left of a chunk is
    // taken before the next chunk starts, so the ring only ever holds one chunk's
    // entries. f(valid, i, index, pattern) is called by all lanes together (from
    // one place: its code exists once), entries of one chunk in index order.
    template <class Keep, class F>
    __device__ __forceinline__ void for_each_vector_entry(const Candidates &cand, uint2 *buf,
                                                          Keep &&keep, F &&f) const
    {
        const u32 lane = lane_id();
        const u64 below = lanes_below();
        RowCursor rc = rows();
        u32 head = 0, pending = 0, cur = 0;
        bool flushing = false;        // the chunk has ended: empty the ring before the next one
        for (;;) {
            while (pending < (u32)kWave && !flushing) {
                if (!rc.open) {
                    if (pending != 0u) { flushing = true; break; }
                    if (!next_chunk(cand, rc)) break;
                    cur = rc.i;
                }
                u32 idx0, bits[4];
                bool valid[4], hit[4];
                load_row(cand, rc, &idx0, bits, valid);
                u64 b[4];
#pragma unroll
                for (u32 e = 0; e < 4; ++e) {
                    hit[e] = valid[e] && keep(bits[e]);
                    b[e] = __ballot(hit[e]);
                }
                if ((b[0] | b[1] | b[2] | b[3]) != 0ull) {
                    u32 p = head + pending + popc64(b[0] & below) + popc64(b[1] & below) +
                            popc64(b[2] & below) + popc64(b[3] & below);
#pragma unroll
                    for (u32 e = 0; e < 4; ++e) {
                        if (hit[e]) { buf[p & (kRowQueueSize - 1u)] = make_uint2(idx0 + e, bits[e]); ++p; }
                    }
                    pending += popc64(b[0]) + popc64(b[1]) + popc64(b[2]) + popc64(b[3]);
                    wave_lds_fence();
                }
            }
            if (pending == 0u) break;             // no chunk left and nothing waiting
            const u32 take = pending < (u32)kWave ? pending : (u32)kWave;
            const bool v = lane < take;
            const uint2 e = v ? buf[(head + lane) & (kRowQueueSize - 1u)] : make_uint2(0u, 0u);
            f(v, cur, e.x, e.y);
            head = (head + take) & (kRowQueueSize - 1u);
            pending -= take;
            if (pending == 0u) flushing = false;
            wave_lds_fence();
        }
    }
};
constexpr u32 kRowQueue = 512;               // ring of one wavefront (ChunkWalk::kRowQueueSize entries)

using UnitWalk = ChunkWalk<kUnitChunksMax>;  // classify / emit: chunks u, u + U, u + 2U, ...

// per-element form of a row callback: f(valid, i, index, pattern) for the four
// elements of a lane, from one call site (the loop is kept rolled)
template <class F>
__device__ __forceinline__ auto each_of_row(F &&f)
{
    return [&f](u32 i, u32 idx0, const u32 (&bits)[4], const bool (&valid)[4]) {
#pragma unroll 1
        for (u32 e = 0; e < 4; ++e) {
            const u32 b = e == 0 ? bits[0] : e == 1 ? bits[1] : e == 2 ? bits[2] : bits[3];
            const bool v = e == 0 ? valid[0] : e == 1 ? valid[1] : e == 2 ? valid[2] : valid[3];
            f(v, i, idx0 + e, b);
        }
    };
}

// ---------------------------------------------------------------------------
// pick: one workgroup finds the bin that holds the r-th largest magnitude
// from the rows the streaming workgroups stored, in two rounds of loads:
// the group sums of all rows (which group holds it, and how many entries lie
// above that group), then that group's bins of all rows.
// ---------------------------------------------------------------------------
constexpr u32 kPickThreads = 1024;

// lane l holds the count of the l-th position from the top (0 beyond the
// last): the position p with #(above p) < need <= #(above p) + count(p), and
// #(above p); found is false when all positions together do not reach need
__device__ __forceinline__ void wave_pick_desc(u32 count, u64 need, u64 above_all, bool *found,
                                               u32 *pos, u64 *above)
{
    const u32 inc = wave_inclusive_sum(count);
    const u64 before = above_all + (inc - count);
    const u64 owner = __ballot(before < need && need <= before + count);
    *found = owner != 0ull;
    const int src = *found ? __ffsll((unsigned long long)owner) - 1 : 0;
    *pos = (u32)src;
    const u32 b_lo = (u32)__builtin_amdgcn_readlane((int)(u32)before, src);
    const u32 b_hi = (u32)__builtin_amdgcn_readlane((int)(u32)(before >> 32), src);
    *above = ((u64)b_hi << 32) | b_lo;
}

__device__ __forceinline__ void
pick_body(const u32 *__restrict__ partials, const u32 *__restrict__ group_sums, u32 n_rows, Geom g,
          EncodeCtl *ctl)
{
    __shared__ u32 gtot[kMaxGroups];
    __shared__ u32 btot[kCoarseSpan];
    __shared__ u32 sel_group, sel_found;
    __shared__ u64 sel_above;
    const Bins bins = ctl->bins;
    const u32 nbins = bins.nfine + kCoarseBins;
    const u32 ngroups = (nbins + kCoarseSpan - 1) / kCoarseSpan;
    const u32 tid = threadIdx.x, lane = lane_id();
    if (tid < kMaxGroups) gtot[tid] = 0u;
    if (tid < kCoarseSpan) btot[tid] = 0u;
    lds_barrier();
    // ---- the group sums of every row, four loads per thread in flight together
    //      (256 rows of 12 groups: one round)
    {
        constexpr u32 kAhead = 4;
        const u32 words = n_rows * ngroups;
        for (u32 i0 = tid; i0 < words; i0 += kAhead * kPickThreads) {
            u32 v[kAhead];
#pragma unroll
            for (u32 q = 0; q < kAhead; ++q) {
                const u32 i = i0 + q * kPickThreads;
                v[q] = i < words ? group_sums[(u64)(i / ngroups) * kMaxGroups + i % ngroups] : 0u;
            }
#pragma unroll
            for (u32 q = 0; q < kAhead; ++q) {
                const u32 i = i0 + q * kPickThreads;
                if (v[q]) atomicAdd(&gtot[i % ngroups], v[q]);
            }
        }
    }
    __syncthreads();
    if (tid < kWave) {
        // groups number at most 36: lane l looks at group ngroups - 1 - l
        static_assert(kMaxGroups <= kWave, "one lane per group");
        const u32 cnt = lane < ngroups ? gtot[ngroups - 1u - lane] : 0u;
        bool found;
        u32 pos;
        u64 above;
        wave_pick_desc(cnt, g.r, 0ull, &found, &pos, &above);
        if (lane == 0) {
            sel_found = found ? 1u : 0u;
            sel_group = found ? ngroups - 1u - pos : 0u;
            sel_above = above;
        }
    }
    lds_barrier();
    bool dense = sel_found == 0u;                  // all rows together hold fewer than r entries
    u32 bin_s = 0;
    u64 before_s = 0;
    if (!dense) {
        // ---- that group's bins of every row: 64 consecutive words per row, sixteen
        //      loads per thread in flight together (256 rows: one round)
        const u32 first_bin = sel_group * kCoarseSpan;
        constexpr u32 kAhead = 16;
        const u32 words = n_rows * kCoarseSpan;
        for (u32 i0 = tid; i0 < words; i0 += kAhead * kPickThreads) {
            u32 v[kAhead];
#pragma unroll
            for (u32 q = 0; q < kAhead; ++q) {
                const u32 i = i0 + q * kPickThreads;
                const u32 b = first_bin + i % kCoarseSpan;
                v[q] = (i < words && b < nbins) ? partials[(u64)(i / kCoarseSpan) * nbins + b] : 0u;
            }
#pragma unroll
            for (u32 q = 0; q < kAhead; ++q) {
                const u32 i = i0 + q * kPickThreads;
                if (v[q]) atomicAdd(&btot[i % kCoarseSpan], v[q]);
            }
        }
        __syncthreads();
        if (tid < kWave) {
            const u32 cnt = btot[kCoarseSpan - 1u - lane];     // bins past nbins stayed 0
            bool found;
            u32 pos;
            u64 above;
            wave_pick_desc(cnt, g.r, sel_above, &found, &pos, &above);
            bin_s = first_bin + (kCoarseSpan - 1u - pos);
            before_s = above;
            if (!found || bin_s >= nbins) dense = true;     // (the group's sum promised otherwise)
        }
    }
    if (tid == 0) {
        u32 bd_lo = 0, bd_hi = 0;
        if (!dense) bin_range(bins, bin_s, &bd_lo, &bd_hi);
        ctl->dense = dense ? 1u : 0u;
        ctl->bd_lo = bd_lo;
        ctl->bd_hi = bd_hi;
        ctl->bd_bits = bd_hi > bd_lo ? 32u - (u32)__clz(bd_hi - bd_lo) : 1u;
        ctl->c_def = before_s;
    }
}

// ---------------------------------------------------------------------------
// classify: walk S; certain members are keyed against the window, entries
// of the deciding bin go to the short list B. Of the deciding bin it also
// leaves the number of entries per chunk and the smallest and largest
// magnitude per workgroup: when the bin turns out to be one long run of equal
// magnitudes (a vector of zeros, of signs, of a few quantisation levels), the
// short list cannot hold it, but the last member is then simply the entry of
// a known rank in index order, which those counts locate.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void
classify_body(Geom g, PhiloxSeed seed, EncodeCtl *ctl, const float *__restrict__ a,
           const u32 *__restrict__ seg_count, const uint2 *__restrict__ s_ent,
           u32 *__restrict__ win_cnt, u32 *__restrict__ bd_cnt, u32 *__restrict__ blk_sure,
           u32 *__restrict__ n_m, u32 *__restrict__ n_b, u32 *__restrict__ blk_bmin,
           u32 *__restrict__ blk_bmax, u64 *__restrict__ m_key, u32 *__restrict__ m_idx,
           u32 *__restrict__ b_mag, u32 *__restrict__ b_idx)
{
    __shared__ u32 cnt_m, cnt_b, cnt_sure, bmin_s, bmax_s;
    __shared__ u32 per_chunk[kWalkWaves][kUnitChunksMax];
    __shared__ u32 per_chunk_b[kWalkWaves][kUnitChunksMax];
    __shared__ uint2 row_queue[kWalkWaves][kRowQueue];
    const u32 wave = threadIdx.x / kWave, lane = lane_id();
    const u32 u = blockIdx.x * kWalkWaves + wave;
    const bool dense = ctl->dense != 0u;
    const u32 bd_lo = ctl->bd_lo, bd_hi = ctl->bd_hi;
    if (dense) {
        if (threadIdx.x == 0) {
            blk_sure[blockIdx.x] = 0u; n_m[blockIdx.x] = 0u; n_b[blockIdx.x] = 0u;
            blk_bmin[blockIdx.x] = 0xFFFFFFFFu; blk_bmax[blockIdx.x] = 0u;
        }
        return;
    }
    const Candidates cand{seg_count, s_ent, a, g.d, g.C, g.U, g.UC, g.cap, false};
    const UnitWalk walk(cand, u < g.U ? u : g.W, g.U, g.W);
    if (threadIdx.x == 0) { cnt_m = 0u; cnt_b = 0u; cnt_sure = 0u; bmin_s = 0xFFFFFFFFu; bmax_s = 0u; }
    if (lane < kUnitChunksMax) { per_chunk[wave][lane] = 0u; per_chunk_b[wave][lane] = 0u; }
    __syncthreads();
    u32 lane_bmin = 0xFFFFFFFFu, lane_bmax = 0u;      // what this lane has already reported

    // entry p of this workgroup's short lists lives at [p][workgroup]: the
    // finalize kernel reads entry p of all workgroups with one coalesced load
    auto slot = [&](u32 p) { return (u64)p * g.G3 + blockIdx.x; };
    const u64 below = lanes_below();
    auto per_entry = [&](bool valid, u32 i, u32 idx, u32 bits) {
        const u32 m = mag_of(bits);
        const bool member = valid && (g.all_members != 0u || m > bd_hi);
        const bool in_bin = valid && !member && m >= bd_lo;
        if (member) {
            bool sure = g.take_all != 0u;
            if (!sure) {
                const u64 key = sample_key(idx, seed);
                if (key < g.K_lo) {
                    sure = true;
                } else if (key <= g.K_hi) {
                    const u32 p = atomicAdd(&cnt_m, 1u);
                    if (p < kListCap) { m_key[slot(p)] = key; m_idx[slot(p)] = idx; }
                }
            }
            if (sure) atomicAdd(&per_chunk[wave][i], 1u);
        }
        if (in_bin) {
            // Entries of the deciding bin are few, or nearly all there is (a run of equal
            // magnitudes): the lanes that are here take their list slots with one addition.
            const u64 here = __ballot(true);
            u32 base = 0;
            if ((here & below) == 0ull) base = atomicAdd(&cnt_b, popc64(here));
            base = (u32)__builtin_amdgcn_readfirstlane((int)base);
            const u32 p = base + popc64(here & below);
            if (p < kListCap) { b_mag[slot(p)] = m; b_idx[slot(p)] = idx; }
            atomicAdd(&per_chunk_b[wave][i], 1u);
            if (m < lane_bmin) { lane_bmin = m; atomicMin(&bmin_s, m); }
            if (m > lane_bmax) { lane_bmax = m; atomicMax(&bmax_s, m); }
        }
    };
    walk.for_each(cand, [&](bool valid, u32 i, u32 idx, u32 bits, u32, u32) {
        per_entry(valid, i, idx, bits);
    });
    if (__builtin_expect(walk.from_vector != 0ull, 0))
        walk.for_each_vector_entry(cand, row_queue[wave],
                                   [&](u32 bits) { return g.all_members != 0u || mag_of(bits) >= bd_lo; },
                                   per_entry);
    __builtin_amdgcn_wave_barrier();
    // certain winners, and entries of the deciding bin, of each of the wavefront's chunks
    u32 mine = 0;
    if (u < g.U && lane < g.UC) {
        const u32 s = u + lane * g.U;
        if (s < g.W) {
            mine = per_chunk[wave][lane];
            win_cnt[s] = mine;
            bd_cnt[s] = per_chunk_b[wave][lane];
        }
    }
    mine = wave_sum(mine);
    if (lane == 0 && mine) atomicAdd(&cnt_sure, mine);
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_sure[blockIdx.x] = cnt_sure;
        n_m[blockIdx.x] = cnt_m < kListCap ? cnt_m : kListCap;
        n_b[blockIdx.x] = cnt_b < kListCap ? cnt_b : kListCap;
        blk_bmin[blockIdx.x] = bmin_s;
        blk_bmax[blockIdx.x] = bmax_s;
        if (cnt_m > kListCap || cnt_b > kListCap) ctl->overflow = 1u;
        if (cnt_m > kListCap) ctl->overflow_m = 1u;
    }
}

// ---------------------------------------------------------------------------
// Radix selection, most significant byte first, over distinct 96-bit strings
// hi:lo (hi 64 bits, lo 32 bits). for_each(f) calls f(hi, lo) for every
// element this thread is responsible for (the elements are split over the
// workgroup in a way that does not change between calls). Returns the
// rank-th smallest string (rank is 1-based). Bytes before first_byte are
// known to be zero in every string. *ok is cleared when fewer than `rank`
// strings exist. Two barriers per byte: the 256-bin histogram rotates through
// three buffers (the next one is cleared while the current one is filled),
// the first wavefront walks the bins and leaves the outcome in a fourth
// buffer for the others. The barriers
// order LDS only; for_each may read global memory but must not depend on
// global writes made by other threads since the last full barrier.
// ---------------------------------------------------------------------------
struct Pair96 {
    u64 hi;
    u32 lo;
};

__device__ __forceinline__ u32 pair_byte(u64 hi, u32 lo, int j /* 0 = most significant */)
{
    return j < 8 ? (u32)(hi >> (56 - 8 * j)) & 0xFFu : (lo >> (24 - 8 * (j - 8))) & 0xFFu;
}

__device__ __forceinline__ bool pair_matches(u64 hi, u32 lo, u64 phi, u32 plo, int nbytes)
{
    // do the first nbytes bytes of hi:lo equal those of phi:plo ?
    if (nbytes <= 0) return true;
    if (nbytes <= 8) return ((hi ^ phi) >> (64 - 8 * nbytes)) == 0ull;
    if (hi != phi) return false;
    return ((lo ^ plo) >> (32 - 8 * (nbytes - 8))) == 0u;
}

template <class ForEach>
__device__ __forceinline__ Pair96 block_select96(ForEach &&for_each, u64 rank, int first_byte,
                                                 u32 (*h)[256] /* 4 buffers */,
                                                 u64 *scratch /* 2 */, bool *ok)
{
    u64 phi = 0;
    u32 plo = 0;
    u64 need = rank;
    int j = first_byte;
    const u32 lane = lane_id();
    *ok = true;
    for (u32 b = threadIdx.x; b < 256u; b += blockDim.x) h[0][b] = 0u;
    lds_barrier();
    u32 cur = 0;
    for (; j < 12; ++j) {
        const u32 nxt = cur == 2u ? 0u : cur + 1u;
        for (u32 b = threadIdx.x; b < 256u; b += blockDim.x) h[nxt][b] = 0u;
        for_each([&](u64 hi, u32 lo) {
            if (pair_matches(hi, lo, phi, plo, j)) atomicAdd(&h[cur][pair_byte(hi, lo, j)], 1u);
        });
        lds_barrier();
        // the first wavefront walks the bins, lane l owning bins 4l .. 4l+3, and leaves
        // the outcome in the fourth buffer for the others (sixteen wavefronts walking
        // them side by side take twice as long as one walk and one more barrier)
        // (the strings number fewer than 2^32, so 32-bit counts do)
        if (threadIdx.x < kWave) {
            u32 c[4];
            u32 mine = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { c[q] = h[cur][4 * lane + q]; mine += c[q]; }
            const u32 inc = wave_inclusive_sum(mine);
            u32 run = inc - mine;
            const bool mine_it = (u64)run < need && need <= (u64)inc;
            const u64 owner = __ballot(mine_it);
            if (owner == 0ull && lane == 0) h[3][3] = 0u;
            if (mine_it) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if ((u64)run < need && need <= (u64)run + c[q]) {
                        h[3][0] = 4 * lane + q;
                        h[3][1] = c[q];
                        h[3][2] = run;
                        h[3][3] = 1u;
                    }
                    run += c[q];
                }
            }
        }
        lds_barrier();
        if (h[3][3] == 0u) { *ok = false; return Pair96{0, 0}; }
        const u32 bin = h[3][0], in_bin = h[3][1], before = h[3][2];
        need -= before;
        if (j < 8) phi |= (u64)bin << (56 - 8 * j);
        else plo |= bin << (24 - 8 * (j - 8));
        cur = nxt;
        if (in_bin == 1u) { ++j; break; }
    }
    if (j < 12) {
        // exactly one string starts with the resolved bytes: fetch the rest of it
        for_each([&](u64 hi, u32 lo) {
            if (pair_matches(hi, lo, phi, plo, j)) { scratch[0] = hi; scratch[1] = lo; }
        });
        lds_barrier();
        phi = scratch[0];
        plo = (u32)scratch[1];
    }
    lds_barrier();
    return Pair96{phi, plo};
}

__device__ __forceinline__ bool pair_le(u64 hi, u32 lo, const Pair96 &p)
{
    return hi < p.hi || (hi == p.hi && lo <= p.lo);
}

// ---------------------------------------------------------------------------
// The same selection spread over the workgroups of one grid (the finalize
// kernel's, at most kWideBlocks, which are resident together). Each workgroup
// histograms its share of the strings in LDS, adds its non-empty bins to the
// pass's 256-bin histogram in the workspace (device-scope atomics), and all
// meet at a barrier; every workgroup then reads the same totals and derives
// the same digit. The barrier is a counter that only grows; a workgroup that
// polls it kWideSpinLimit times in vain gives up, which ends the kernel with
// an error flag instead of a hang (the others give up in turn).
// ---------------------------------------------------------------------------
struct Wide {
    WideScratch *ws;
    u32 nblocks;
    u32 epoch;          // barriers passed
    u32 pass;           // histogram / fetch slots used
    bool alive;         // false once a barrier timed out
    u32 spin_limit;     // polls before a workgroup gives up at a barrier
};

// Everything the workgroups exchange goes through device-scope atomic
// operations (additions to the histograms, atomic stores of the few words
// workgroup 0 reads at the end, atomic loads on the reading side), which are
// carried out where all compute units see them. The barrier therefore only has
// to order them: every thread waits until its own operations are acknowledged
// (a workgroup-scope release does that) before its workgroup checks in. A
// device-scope fence per thread, which writes back and invalidates the L2 of
// the XCD, made a barrier of 256 workgroups cost ~100 us.
__device__ __forceinline__ bool grid_barrier(Wide &w, u32 *lds_flag)
{
    if (!w.alive) return false;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    ++w.epoch;
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(&w.ws->arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const u32 target = w.epoch * w.nblocks;
        u32 polls = 0;
        bool ok = true;
        while (__hip_atomic_load(&w.ws->arrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(32);
            if (++polls > w.spin_limit) { ok = false; break; }
        }
        *lds_flag = ok ? 1u : 0u;
    }
    __syncthreads();
    w.alive = *lds_flag != 0u;
    __syncthreads();
    return w.alive;
}

// What the selection over the grid settles: the first `bytes` bytes of the
// rank-th smallest string (the rest of hi:lo is zero). With bytes < 12 exactly
// ONE string starts with them, so "at or below the selected string" is the
// same as "at or below these bytes followed by ones" (bound()), and nobody has
// to go and fetch the rest before the next pass can start; is() recognises the
// selected string itself when a later pass comes across it.
struct Selected {
    u64 hi;
    u32 lo;
    int bytes;
    __device__ __forceinline__ Pair96 bound() const
    {
        if (bytes >= 12) return Pair96{hi, lo};
        if (bytes > 8) return Pair96{hi, lo | ((1u << (32 - 8 * (bytes - 8))) - 1u)};
        if (bytes == 8) return Pair96{hi, 0xFFFFFFFFu};
        return Pair96{hi | ((1ull << (64 - 8 * bytes)) - 1ull), 0xFFFFFFFFu};
    }
    __device__ __forceinline__ bool is(u64 shi, u32 slo) const { return pair_matches(shi, slo, hi, lo, bytes); }
};

// Before the first barrier the workgroups of the grid make sure that ALL of
// them are resident: every workgroup checks in; the last to arrive decides
// "go", a workgroup that has polled kWideCheckInLimit times in vain decides
// "abort" (compare-and-swap: one decision stands), and everybody waits for the
// decision. After "go" every workgroup is running, so the later barriers
// cannot wait for one that was never scheduled (two grids of two streams, each
// holding half of the compute units, would otherwise wait for each other until
// the poll limit). After "abort" nothing has been computed yet: the caller
// falls back to the selection by one workgroup. Counts as the first barrier.
__device__ __forceinline__ bool grid_check_in(Wide &w, u32 *lds_flag)
{
    __syncthreads();
    ++w.epoch;
    if (threadIdx.x == 0) {
        const u32 mine = __hip_atomic_fetch_add(&w.ws->arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
        u32 expected = 0u;
        if (mine == w.nblocks)
            __hip_atomic_compare_exchange_strong(&w.ws->decision, &expected, kWideGo, __ATOMIC_RELAXED,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        u32 polls = 0, d = 0;
        while ((d = __hip_atomic_load(&w.ws->decision, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == 0u) {
            __builtin_amdgcn_s_sleep(32);
            if (++polls == kWideCheckInLimit) {
                expected = 0u;
                __hip_atomic_compare_exchange_strong(&w.ws->decision, &expected, kWideAbort,
                                                     __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
            }
            if (polls > kWideSpinLimit) { d = kWideAbort; break; }   // (cannot happen: somebody decides)
        }
        *lds_flag = d == kWideGo ? 1u : 0u;
    }
    __syncthreads();
    const bool go = *lds_flag != 0u;
    __syncthreads();
    return go;
}

// for_each(f) calls f(valid, hi, lo) for every string of this workgroup's
// share, ALL lanes of a wavefront together (valid says whether the lane holds
// one). *less_hi receives the number of strings whose high 64 bits are below
// the result's. h: 4 x 256 words of LDS.
template <class ForEach>
__device__ __forceinline__ Selected grid_select96(ForEach &&for_each, u64 rank, int first_byte, Wide &w,
                                                  u32 (*h)[256], u64 *less_hi, bool *ok)
{
    u64 phi = 0;
    u32 plo = 0;
    u64 need = rank;
    int j = first_byte;
    const u32 lane = lane_id();
    *ok = true;
    *less_hi = 0;
    for (; j < 12; ++j) {
        for (u32 b = threadIdx.x; b < 256u; b += blockDim.x) h[0][b] = 0u;
        lds_barrier();
        for_each([&](bool valid, u64 hi, u32 lo) {
            const bool on = valid && pair_matches(hi, lo, phi, plo, j);
            const u32 digit = pair_byte(hi, lo, j);
            // neighbouring strings often share the digit (runs of equal magnitudes): when all
            // of a wavefront's do, one addition serves them
            const u64 m = __ballot(on);
            if (m == 0ull) return;
            const int src = __ffsll((unsigned long long)m) - 1;
            const u32 first = (u32)__builtin_amdgcn_readlane((int)digit, src);
            if (__ballot(on && digit == first) == m) {
                if ((int)lane == src) atomicAdd(&h[0][first], popc64(m));
            } else if (on) {
                atomicAdd(&h[0][digit], 1u);
            }
        });
        lds_barrier();
        if (w.pass >= kWidePasses) { *ok = false; return Selected{0, 0, 12}; }
        u32 *gh = w.ws->hist[w.pass];
        for (u32 b = threadIdx.x; b < 256u; b += blockDim.x)
            if (h[0][b]) atomicAdd(&gh[b], h[0][b]);
        if (!grid_barrier(w, &h[3][4])) { *ok = false; return Selected{0, 0, 12}; }
        if (threadIdx.x < kWave) {
            u32 c[4];
            u32 mine = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                c[q] = __hip_atomic_load(&gh[4 * lane + q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                mine += c[q];
            }
            const u32 inc = wave_inclusive_sum(mine);
            u32 run = inc - mine;
            const bool mine_it = (u64)run < need && need <= (u64)inc;
            const u64 owner = __ballot(mine_it);
            if (owner == 0ull && lane == 0) h[3][3] = 0u;
            if (mine_it) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if ((u64)run < need && need <= (u64)run + c[q]) {
                        h[3][0] = 4 * lane + q;
                        h[3][1] = c[q];
                        h[3][2] = run;
                        h[3][3] = 1u;
                    }
                    run += c[q];
                }
            }
        }
        lds_barrier();
        ++w.pass;
        if (h[3][3] == 0u) { *ok = false; return Selected{0, 0, 12}; }
        const u32 bin = h[3][0], in_bin = h[3][1], before = h[3][2];
        lds_barrier();
        need -= before;
        if (j < 8) { phi |= (u64)bin << (56 - 8 * j); *less_hi += before; }
        else plo |= bin << (24 - 8 * (j - 8));
        if (in_bin == 1u) { ++j; break; }
    }
    return Selected{phi, plo, j};
}

// ---------------------------------------------------------------------------
// finalize: turns the short lists into the two cut points and the output
// offset of every chunk (workgroup 0; the others leave at once), or, when the
// counts left by classify show that the lists cannot decide and the vector is
// long, runs the exact selection over all candidates on all its workgroups.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void
finalize_body(Geom g, PhiloxSeed seed, EncodeCtl *ctl, WideScratch *wide_ws,
           const float *__restrict__ a,
           const u32 *__restrict__ seg_count, const uint2 *__restrict__ s_ent,
           u32 *win_cnt, const u32 *__restrict__ bd_cnt, const u32 *__restrict__ blk_sure,
           const u32 *__restrict__ n_m, const u32 *__restrict__ n_b,
           const u32 *__restrict__ blk_bmin, const u32 *__restrict__ blk_bmax,
           const u64 *__restrict__ m_key, const u32 *__restrict__ m_idx,
           const u32 *__restrict__ b_mag, const u32 *__restrict__ b_idx, u64 *dm_key,
           u32 *dm_idx, u64 *db_key, u32 *db_idx, u32 *__restrict__ chunk_base)
{
    static_assert(kMaxWalkBlocks <= (u32)kFinThreads, "one thread per classify workgroup");
    __shared__ u32 h[4][256];
    __shared__ u32 scan32[kSlabs * kFinWaves + 1];
    __shared__ u64 scratch[2];
    __shared__ u64 st_b_key[kStageB];
    __shared__ u32 st_b_idx[kStageB];
    __shared__ u64 st_m_key[kStageM];
    __shared__ u32 st_m_idx[kStageM];
    __shared__ u32 extra_m, sure_extra;
    __shared__ unsigned long long gt_extra;
    __shared__ u32 run_chunk, run_before, run_index, run_found;
    __shared__ u32 run_sure[kFinWaves][kUnitChunksMax];

    const u32 tid = threadIdx.x;
    const u32 wave = tid / kWave, lane = lane_id();
    const bool dense = ctl->dense != 0u;
    Candidates cand{seg_count, s_ent, a, g.d, g.C, g.U, g.UC, g.cap, dense};
    // every candidate, split wavefront by chunk; f(index, pattern, chunk)
    auto each_s = [&](auto &&f) {
        // kWave consecutive chunks per wavefront at a time: their sizes in one round of
        // loads, then their entries as one flat sequence, four iterations fetched together
        for (u32 first = wave * kWave; first < g.W; first += kFinWaves * kWave) {
            const ChunkWalk<kWave> walk(cand, first, 1u, g.W);
            walk.for_each(cand, [&](bool valid, u32 i, u32 idx, u32 bits, u32, u32) {
                if (valid) f(idx, bits, first + i);
            });
            auto of_row = [&](bool valid, u32 i, u32 idx, u32 bits) {
                if (valid) f(idx, bits, first + i);
            };
            walk.for_each_vector_row(cand, each_of_row(of_row));
        }
    };

    // ---- everything the short-list path needs, fetched in one round ------
    const bool in_grid = tid < g.G3;
    const u32 vm = in_grid ? n_m[tid] : 0u, vb = in_grid ? n_b[tid] : 0u;
    const u32 vs = in_grid ? blk_sure[tid] : 0u;
    const u32 bd_lo = ctl->bd_lo, bd_hi = ctl->bd_hi, bd_bits = ctl->bd_bits;
    const u64 c_def = ctl->c_def;
    const bool overflow = ctl->overflow != 0u, overflow_m = ctl->overflow_m != 0u;
    if (tid == 0) { extra_m = 0u; sure_extra = 0u; gt_extra = 0ull; run_found = 0u; }
    // The three totals (every workgroup of the grid needs them to decide whether
    // it stays) and, from the same partial sums, where this thread's classify
    // workgroup's entries start in the two lists: one exchange, every wavefront
    // adds up the sixteen partial sums for itself.
    u32 n_m0, n_bd, em, eb;
    u64 sure_walk;
    {
        const u32 im = wave_inclusive_sum(vm), ib = wave_inclusive_sum(vb), wsure = wave_sum(vs);
        if (lane == kWave - 1) { scan32[wave] = im; scan32[kFinWaves + wave] = ib; scan32[2 * kFinWaves + wave] = wsure; }
        static_assert(3 * kFinWaves <= kSlabs * kFinWaves + 1, "room for three partial sums per wavefront");
        static_assert(kFinWaves <= kWave, "one lane per wavefront's partial sum");
        lds_barrier();
        const u32 pm = lane < kFinWaves ? scan32[lane] : 0u;
        const u32 pb = lane < kFinWaves ? scan32[kFinWaves + lane] : 0u;
        n_m0 = wave_sum(pm);
        n_bd = wave_sum(pb);
        sure_walk = wave_sum(lane < kFinWaves ? scan32[2 * kFinWaves + lane] : 0u);
        em = wave_sum(lane < wave ? pm : 0u) + im - vm;
        eb = wave_sum(lane < wave ? pb : 0u) + ib - vb;
        lds_barrier();
    }

    const u64 need2 = g.r - c_def;
    u32 err = 0, path = 0;
    bool have_t = false, have_k = false, ok = true;
    u32 T = 0, I_star = 0, J_star = 0xFFFFFFFFu, n_mm = 0;
    u64 K_star = ~0ull, count_greater = 0;

    if (g.all_members) {
        // r == d: the "threshold" is the whole vector; only the key cut is found
        have_t = true;
        T = 0u;
        I_star = 0xFFFFFFFFu;
    }
    const bool lists = !dense && !overflow && (g.all_members || (c_def < g.r && need2 <= n_bd));
    // The list B overflowed but M did not, and every entry of the deciding bin has
    // the same magnitude: the last member is the need2-th of them in index order.
    bool tie_run = false;
    if (__builtin_expect(!dense && overflow && !overflow_m && !g.all_members && c_def < g.r, 0)) {
        const u32 vmin = in_grid ? blk_bmin[tid] : 0xFFFFFFFFu, vmax = in_grid ? blk_bmax[tid] : 0u;
        const u32 lo = wave_min(vmin), hi = wave_max(vmax);
        if (lane == 0) { scan32[wave] = lo; scan32[kFinWaves + wave] = hi; }
        lds_barrier();
        const u32 all_lo = wave_min(lane < kFinWaves ? scan32[lane] : 0xFFFFFFFFu);
        const u32 all_hi = wave_max(lane < kFinWaves ? scan32[kFinWaves + lane] : 0u);
        lds_barrier();
        tie_run = all_lo == all_hi;
        if (tie_run) T = all_lo;
    }
    // ---- many workgroups or one? Every workgroup of the grid decides alike,
    //      from what classify and pick left: the lists cannot give the
    //      threshold (the estimate kept too little; the deciding bin crowded by
    //      several magnitudes), or the key window certainly missed.
    bool wide = false;
    if (gridDim.x > 1u) {
        const bool slow_t = !g.all_members && !lists && !tie_run;
        bool slow_k = false;
        if (!g.take_all && !tie_run) {
            const u64 from_b = (g.all_members || !lists) ? 0ull : (need2 < n_bd ? need2 : (u64)n_bd);
            slow_k = dense || overflow_m || (g.all_members && overflow) || sure_walk >= g.k ||
                     sure_walk + n_m0 + from_b < g.k;
        }
        wide = slow_t || slow_k;
        if (!wide && blockIdx.x != 0u) return;
    }
    if (__builtin_expect(wide, 0)) {
        // ---- exact selection over all candidates, on all workgroups of the grid
        Wide w{wide_ws, gridDim.x, 0u, 0u, true, kWideSpinLimit};
        if (g.force_abort != 0u || !grid_check_in(w, &h[3][4])) {
            // the grid's workgroups cannot be resident together right now (another
            // stream's grid holds compute units and waits as well): nothing has been
            // done yet, workgroup 0 runs the selection alone below
            if (blockIdx.x != 0u) return;
            wide = false;
        }
    }
    if (__builtin_expect(wide, 0)) {
        // (diagnostics: with no patience at all the barriers time out, the kernel ends
        // with the error flag set and every workgroup still leaves normally)
        Wide w{wide_ws, gridDim.x, 1u, 0u, true, g.force_timeout != 0u ? 0u : kWideSpinLimit};
        // r == d: S only holds the coordinates inside the key window, which
        // missed: the vector itself is walked, here and by the emit kernel
        if (g.all_members) cand.dense = true;
        const bool vec16 = (reinterpret_cast<uintptr_t>(a) & 15u) == 0;
        const u32 n_waves = gridDim.x * kFinWaves;
        // f(valid, index, pattern) for every entry of this workgroup's chunks, all lanes
        // together; done(s) after the last entry of chunk s. Wavefront v of the grid takes
        // chunks v, v + n_waves, ...; a chunk read from the vector is streamed with
        // 16-byte loads, four rows in flight.
        auto wide_each = [&](auto &&f, auto &&done) {
            for (u32 sc = blockIdx.x * kFinWaves + wave; sc < g.W; sc += n_waves) {
                bool fv = false;
                const u32 n_e = cand.count(sc, &fv);
                if (!fv) {
                    for (u32 j0 = 0; j0 < n_e; j0 += kWave) {
                        const u32 j = j0 + lane;
                        u32 idx = 0, bits = 0;
                        if (j < n_e) cand.entry(sc, j, false, &idx, &bits);
                        f(j < n_e, idx, bits);
                    }
                } else {
                    const u64 c0 = (u64)sc * g.C;
                    u32 j0 = 0;
                    if (vec16) {
                        for (; j0 + 4 * kChunkQuantum <= n_e; j0 += 4 * kChunkQuantum) {
                            const f32x4 *p4 = reinterpret_cast<const f32x4 *>(a + c0 + j0) + lane;
                            f32x4 v[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q) v[q] = p4[q * kWave];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const u32 i0 = (u32)(c0 + j0) + (u32)q * kChunkQuantum + 4u * lane;
                                f(true, i0, __float_as_uint(v[q].x));
                                f(true, i0 + 1u, __float_as_uint(v[q].y));
                                f(true, i0 + 2u, __float_as_uint(v[q].z));
                                f(true, i0 + 3u, __float_as_uint(v[q].w));
                            }
                        }
                    }
                    for (; j0 < n_e; j0 += kWave) {
                        const u32 j = j0 + lane;
                        const u32 bits = j < n_e ? __float_as_uint(a[c0 + j]) : 0u;
                        f(j < n_e, (u32)(c0 + j), bits);
                    }
                }
                done(sc);
            }
        };
        auto nothing = [](u32) {};
        path = 1u | 8u;
        // where whoever comes across a selected string in a later pass leaves it whole
        u64 *found_t = w.ws->found[kWidePasses - 2], *found_k = w.ws->found[kWidePasses - 1];
        const bool in_bin_only = !g.all_members && !cand.dense;
        const u32 top = in_bin_only ? bd_hi : 0x7FFFFFFFu;
        Selected sel_t{0ull, 0u, 12}, sel_k{0ull, 0u, 12};
        Pair96 tbound{~0ull, 0xFFFFFFFFu}, kbound{~0ull, 0xFFFFFFFFu};
        if (!g.all_members) {
            // the r-th (magnitude desc, index asc): inside the deciding bin when pick found
            // one, over the whole vector when the estimate had kept too little
            auto each_mag = [&](auto &&f2) {
                wide_each([&](bool valid, u32 idx, u32 bits) {
                    const u32 m = mag_of(bits);
                    const bool on = valid && (!in_bin_only || (m >= bd_lo && m <= bd_hi));
                    f2(on, (u64)(top - (on ? m : top)), idx);
                }, nothing);
            };
            u64 less = 0;
            sel_t = grid_select96(each_mag, in_bin_only ? need2 : g.r,
                                  in_bin_only ? (64 - (int)bd_bits) / 8 : 4, w, h, &less, &ok);
            if (!ok) err |= kErrSelect;
            tbound = sel_t.bound();
            count_greater = (in_bin_only ? c_def : 0ull) + less;
        }
        // members: above the deciding bin, or at or below the selected string in
        // (magnitude desc, index asc) order
        auto is_member_w = [&](u32 idx, u32 bits) {
            if (g.all_members != 0u) return true;
            const u32 m = mag_of(bits);
            if (m > top) return true;
            if (in_bin_only && m < bd_lo) return false;
            return pair_le((u64)(top - m), idx, tbound);
        };
        if (!g.take_all && w.alive) {
            auto each_key = [&](auto &&f2) {
                wide_each([&](bool valid, u32 idx, u32 bits) {
                    const bool on = valid && is_member_w(idx, bits);
                    f2(on, on ? sample_key(idx, seed) : 0ull, idx);
                }, nothing);
            };
            u64 less = 0;
            bool ok_k = true;
            sel_k = grid_select96(each_key, g.k, 0, w, h, &less, &ok_k);
            if (!ok_k) err |= kErrSelect;
            kbound = sel_k.bound();
        }
        // winners per chunk (every chunk's counter is written: what classify left is
        // stale); the same pass leaves the two selected strings whole for workgroup 0
        if (w.alive) {
            u32 mine = 0;
            wide_each([&](bool valid, u32 idx, u32 bits) {
                if (!valid || !is_member_w(idx, bits)) return;
                const u32 m = mag_of(bits);
                if (sel_t.bytes < 12 && m <= top && sel_t.is((u64)(top - m), idx)) {
                    __hip_atomic_store(&found_t[0], (u64)(top - m), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&found_t[1], (u64)idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (g.take_all != 0u) { ++mine; return; }
                const u64 key = sample_key(idx, seed);
                if (!pair_le(key, idx, kbound)) return;
                ++mine;
                if (sel_k.bytes < 12 && sel_k.is(key, idx)) {
                    __hip_atomic_store(&found_k[0], key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&found_k[1], (u64)idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }, [&](u32 sc) {
                const u32 total = wave_sum(mine);
                if (lane == 0)
                    __hip_atomic_store(&win_cnt[sc], total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                mine = 0;
            });
            grid_barrier(w, &h[3][4]);
        }
        if (w.alive && blockIdx.x == 0u) {
            Pair96 ts{sel_t.hi, sel_t.lo}, ks{sel_k.hi, sel_k.lo};
            if (sel_t.bytes < 12) {
                ts.hi = __hip_atomic_load(&found_t[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ts.lo = (u32)__hip_atomic_load(&found_t[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (sel_k.bytes < 12) {
                ks.hi = __hip_atomic_load(&found_k[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ks.lo = (u32)__hip_atomic_load(&found_k[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (!g.all_members) { T = top - (u32)ts.hi; I_star = ts.lo; }
            if (!g.take_all) { K_star = ks.hi; J_star = ks.lo; }
        }
        if (!w.alive) err |= kErrBarrier;
        if (blockIdx.x != 0u) return;
        have_t = true;
        have_k = true;
        if (g.all_members && tid == 0) ctl->dense = 1u;
    }

    // The short-list path. It is compiled twice: once with both lists in LDS
    // (the usual case; the compiler then knows the address space of every list
    // access and overlaps the loads that fill the lists) and once with the
    // lists wherever they fit.
    auto short_lists = [&](u64 *bk, u32 *bi, u64 *mk, u32 *mi, auto all_lds_tag) {
        constexpr bool kAllLds = decltype(all_lds_tag)::value;
        const u32 n_b_use = lists ? n_bd : 0u;
        const bool m_lds = kAllLds || (lists && n_m0 + n_b_use <= kStageM);
        const u32 m_cap = m_lds ? kStageM : 2u * g.G3 * kListCap;
        auto barrier = [&] { if (kAllLds) lds_barrier(); else __syncthreads(); };
        // Entry j of classify workgroup t lives at [j][t]. First every thread
        // notes where the entries of its workgroup are (no memory latency in
        // that loop), then the entries are fetched position by position, all
        // loads of a thread in flight together.
        if (lists) for (u32 j = 0; j < vb; ++j) bi[eb + j] = j * g.G3 + tid;
        for (u32 j = 0; j < vm; ++j) mi[em + j] = j * g.G3 + tid;
        barrier();
        if (kAllLds) {
            constexpr u32 kB = kStageB / kFinThreads, kM = kStageM / kFinThreads;
            u32 b_m[kB], b_i[kB], m_i[kM];
            u64 m_k[kM];
#pragma unroll
            for (u32 q = 0; q < kB; ++q) {
                const u32 p = q * kFinThreads + tid;
                if (p < n_b_use) { const u32 at = bi[p]; b_m[q] = b_mag[at]; b_i[q] = b_idx[at]; }
            }
#pragma unroll
            for (u32 q = 0; q < kM; ++q) {
                const u32 p = q * kFinThreads + tid;
                if (p < n_m0) { const u32 at = mi[p]; m_k[q] = m_key[at]; m_i[q] = m_idx[at]; }
            }
#pragma unroll
            for (u32 q = 0; q < kB; ++q) {
                const u32 p = q * kFinThreads + tid;
                if (p < n_b_use) { bk[p] = (u64)(bd_hi - b_m[q]); bi[p] = b_i[q]; }
            }
#pragma unroll
            for (u32 q = 0; q < kM; ++q) {
                const u32 p = q * kFinThreads + tid;
                if (p < n_m0) { mk[p] = (m_k[q] - g.K_lo) << g.k_nlz; mi[p] = m_i[q]; }
            }
        } else {
            for (u32 p = tid; p < n_b_use; p += kFinThreads) {
                const u32 at = bi[p];
                bk[p] = (u64)(bd_hi - b_mag[at]);
                bi[p] = b_idx[at];
            }
            for (u32 p = tid; p < n_m0; p += kFinThreads) {
                const u32 at = mi[p];
                mk[p] = (m_key[at] - g.K_lo) << g.k_nlz;
                mi[p] = m_idx[at];
            }
        }
        barrier();
        // (in LDS a thread's entries, two at most, stay in registers over the rounds)
        constexpr u32 kB = kAllLds ? kStageB / kFinThreads : 1u;
        u64 rb_k[kB];
        u32 rb_i[kB];
        if (kAllLds) {
#pragma unroll
            for (u32 q = 0; q < kB; ++q) {
                const u32 p = q * kFinThreads + tid;
                rb_k[q] = p < n_bd ? bk[p] : 0ull;
                rb_i[q] = p < n_bd ? bi[p] : 0u;
            }
        }
        auto each_b = [&](auto &&f) {
            if (kAllLds) {
#pragma unroll
                for (u32 q = 0; q < kB; ++q)
                    if (q * kFinThreads + tid < n_bd) f(rb_k[q], rb_i[q]);
            } else {
                for (u32 p = tid; p < n_bd; p += kFinThreads) f(bk[p], bi[p]);
            }
        };
        Pair96 tb{0ull, 0u};
        if (__builtin_expect(tie_run, 0)) {
            // ---- the chunk that holds the need2-th entry of the run: thread t
            //      adds up the counts of chunks 32t .. 32t+31 ---------------------
            path = 4;
            constexpr u32 kPer = kTargetChunks / kFinThreads;
            static_assert(kPer % 4 == 0, "whole 16-byte groups of counters per thread");
            u32 mine = 0;
#pragma unroll
            for (u32 q = 0; q < kPer / 4; ++q) {
                const u32 s = tid * kPer + 4u * q;
                uint4 v = make_uint4(0u, 0u, 0u, 0u);
                if (s < g.W) v = reinterpret_cast<const uint4 *>(bd_cnt)[s / 4];
                mine += v.x + (s + 1 < g.W ? v.y : 0u) + (s + 2 < g.W ? v.z : 0u) +
                        (s + 3 < g.W ? v.w : 0u);
            }
            // (the entries of the bin number at most d < 2^32)
            const u32 before = block_exclusive_sum(mine, scan32);
            if ((u64)before < need2 && need2 <= (u64)before + mine) {
                run_chunk = tid * kPer;          // first of the kPer chunks that hold it
                run_before = before;
                run_found = 1u;
            }
            lds_barrier();
            if (wave == 0 && run_found != 0u) {
                // the counters of those chunks again, one per lane
                static_assert(kPer <= kWave, "one lane per counter");
                const u32 s0 = run_chunk, b0 = run_before;
                const u32 s = s0 + lane;
                const u32 c = (lane < kPer && s < g.W) ? bd_cnt[s] : 0u;
                const u32 inc = wave_inclusive_sum(c);
                if ((u64)b0 + (inc - c) < need2 && need2 <= (u64)b0 + inc) {
                    run_chunk = s;
                    run_before = b0 + (inc - c);
                }
            }
            lds_barrier();
            ok = run_found != 0u;
            if (ok) {
                // ---- the entry of that rank inside the chunk, 1024 entries a round
                const u32 sc = run_chunk;
                const u32 want = (u32)(need2 - run_before);      // 1-based, among the chunk's
                bool sc_vec = false;
                const u32 n_e = cand.count(sc, &sc_vec);
                lds_barrier();
                if (tid == 0) run_found = 0u;
                u32 seen = 0;
                for (u32 j0 = 0; j0 < n_e && seen < want; j0 += kFinThreads) {
                    const u32 j = j0 + tid;
                    u32 idx = 0, bits = 0;
                    if (j < n_e) cand.entry(sc, j, sc_vec, &idx, &bits);
                    const u32 m = mag_of(bits);
                    const u32 flag = (j < n_e && m >= bd_lo && m <= bd_hi) ? 1u : 0u;
                    const u32 excl = block_exclusive_sum(flag, scan32);
                    const u32 round_total = scan32[kFinWaves];
                    if (flag && seen + excl + 1u == want) { run_index = idx; run_found = 1u; }
                    seen += round_total;
                    lds_barrier();
                }
                ok = run_found != 0u;
                I_star = run_index;
            }
            if (!ok) { T = 0; path = 0; }
        } else if (!g.all_members) {
            // ---- exact threshold inside the deciding bin --------------------
            tb = block_select96(each_b, need2, (64 - (int)bd_bits) / 8, h, scratch, &ok);
        }
        if (ok) {
            have_t = true;
            if (lists && !g.all_members) {
                T = bd_hi - (u32)tb.hi;
                I_star = tb.lo;
            }
            // ---- members of the deciding bin join the key lists; the atomics
            //      on the chunk counters are left in flight --------------------
            // join(idx, on_sure): idx is a member; its key decides between "certain
            // winner" (on_sure is called), the key list M, or nothing
            auto join = [&](u32 idx, auto &&on_sure) {
                if (g.take_all != 0u) { on_sure(); return; }
                const u64 key = sample_key(idx, seed);
                if (key < g.K_lo) {
                    on_sure();
                } else if (key <= g.K_hi) {
                    const u32 q = atomicAdd(&extra_m, 1u);
                    if (n_m0 + q < m_cap) {
                        mk[n_m0 + q] = (key - g.K_lo) << g.k_nlz;
                        mi[n_m0 + q] = idx;
                    }
                }
            };
            u32 my_gt = 0;
            if (__builtin_expect(lists, 1)) {
                each_b([&](u64 hi, u32 idx) {
                    if (hi < tb.hi) ++my_gt;
                    if (pair_le(hi, idx, tb))
                        join(idx, [&] { atomicAdd(&win_cnt[idx / g.C], 1u); atomicAdd(&sure_extra, 1u); });
                });
            } else {
                // the run's members: its entries up to index I*, all in chunks 0 .. run_chunk.
                // They may be many per chunk: certain winners are counted per chunk in LDS
                // and reach the chunk's counter as one addition.
                const u32 s_end = run_chunk + 1u;
                u32 my_sure = 0;
                for (u32 first = wave * kUnitChunksMax; first < s_end; first += kFinWaves * kUnitChunksMax) {
                    if (lane < kUnitChunksMax) run_sure[wave][lane] = 0u;
                    __builtin_amdgcn_wave_barrier();
                    const UnitWalk walk(cand, first, 1u, s_end);
                    auto run_member = [&](bool valid, u32 i, u32 idx, u32 bits) {
                        const u32 m = mag_of(bits);
                        if (valid && m >= bd_lo && m <= bd_hi && idx <= I_star)
                            join(idx, [&] { atomicAdd(&run_sure[wave][i], 1u); ++my_sure; });
                    };
                    walk.for_each(cand, [&](bool valid, u32 i, u32 idx, u32 bits, u32, u32) {
                        run_member(valid, i, idx, bits);
                    });
                    walk.for_each_vector_row(cand, each_of_row(run_member));
                    __builtin_amdgcn_wave_barrier();
                    if (lane < kUnitChunksMax && first + lane < s_end && run_sure[wave][lane])
                        atomicAdd(&win_cnt[first + lane], run_sure[wave][lane]);
                    __builtin_amdgcn_wave_barrier();
                }
                my_sure = wave_sum(my_sure);
                if (lane == 0 && my_sure) atomicAdd(&sure_extra, my_sure);
            }
            if (my_gt) atomicAdd(&gt_extra, (unsigned long long)my_gt);
            barrier();
            count_greater = c_def + gt_extra;
            n_mm = n_m0 + extra_m;
            if (__builtin_expect(tie_run && n_mm <= kStageM && n_mm <= m_cap, 0)) {
                // short after all: the selection below reads it several times, from LDS then
                for (u32 p = tid; p < n_mm; p += kFinThreads) { st_m_key[p] = mk[p]; st_m_idx[p] = mi[p]; }
                mk = st_m_key;
                mi = st_m_idx;
                lds_barrier();
            }
            const u64 c_klo = sure_walk + sure_extra;
            if (g.take_all) {
                have_k = true;
            } else if (n_mm <= m_cap && c_klo < g.k && g.k - c_klo <= n_mm) {
                // (in LDS a thread's entries, four at most, stay in registers over the rounds)
                constexpr u32 kM = kAllLds ? kStageM / kFinThreads : 1u;
                u64 rm_k[kM];
                u32 rm_i[kM];
                if (kAllLds) {
#pragma unroll
                    for (u32 q = 0; q < kM; ++q) {
                        const u32 p = q * kFinThreads + tid;
                        rm_k[q] = p < n_mm ? mk[p] : 0ull;
                        rm_i[q] = p < n_mm ? mi[p] : 0u;
                    }
                }
                auto each_m = [&](auto &&f) {
                    if (kAllLds) {
#pragma unroll
                        for (u32 q = 0; q < kM; ++q)
                            if (q * kFinThreads + tid < n_mm) f(rm_k[q], rm_i[q]);
                    } else {
                        for (u32 p = tid; p < n_mm; p += kFinThreads) f(mk[p], mi[p]);
                    }
                };
                const Pair96 kb = block_select96(each_m, g.k - c_klo, 0, h, scratch, &ok);
                if (ok) {
                    have_k = true;
                    K_star = (kb.hi >> g.k_nlz) + g.K_lo;
                    J_star = kb.lo;
                    each_m([&](u64 key, u32 idx) {
                        if (pair_le(key, idx, kb)) atomicAdd(&win_cnt[idx / g.C], 1u);
                    });
                }
            }
        }
    };
    if (!wide && (lists || tie_run)) {
        const u32 n_b_use = lists ? n_bd : 0u;
        const bool b_lds = n_b_use <= kStageB;
        // (a run of equal magnitudes may add any number of keys: the large array then)
        const bool m_lds = lists && n_m0 + n_b_use <= kStageM;
        if (b_lds && m_lds)
            short_lists(st_b_key, st_b_idx, st_m_key, st_m_idx, std::true_type{});
        else
            short_lists(b_lds ? st_b_key : db_key, b_lds ? st_b_idx : db_idx,
                        m_lds ? st_m_key : dm_key, m_lds ? st_m_idx : dm_idx, std::false_type{});
    }

    if (g.all_members && !have_k) {
        // r == d and the key window missed (or a short list overflowed): the
        // candidates are only the coordinates inside the window, so the exact
        // selection below walks the vector itself, and so does the emit kernel
        cand.dense = true;
        if (tid == 0) ctl->dense = 1u;
    }
    if (!have_t) {
        // ---- exact threshold by selection over all candidates -----------
        path |= 1u;
        auto each_mag = [&](auto &&f) {
            each_s([&](u32 idx, u32 bits, u32) { f((u64)(0x7FFFFFFFu - mag_of(bits)), idx); });
        };
        const Pair96 tb = block_select96(each_mag, g.r, 4, h, scratch, &ok);
        if (!ok) err |= kErrSelect;
        T = 0x7FFFFFFFu - (u32)tb.hi;
        I_star = tb.lo;
        u32 my_gt = 0;
        each_s([&](u32, u32 bits, u32) { if (mag_of(bits) > T) ++my_gt; });
        count_greater = block_sum(my_gt, scan32);
    }
    auto is_member = [&](u32 idx, u32 bits) {
        const u32 m = mag_of(bits);
        return m > T || (m == T && idx <= I_star);
    };
    if (!have_k) {
        // ---- exact key cut and winners per chunk by selection over all candidates
        path |= 1u;
        __syncthreads();
        for (u32 s = tid; s < g.W; s += kFinThreads) win_cnt[s] = 0u;
        if (!g.take_all) {
            auto each_key = [&](auto &&f) {
                each_s([&](u32 idx, u32 bits, u32) {
                    if (is_member(idx, bits)) f(sample_key(idx, seed), idx);
                });
            };
            const Pair96 kb = block_select96(each_key, g.k, 0, h, scratch, &ok);
            if (!ok) err |= kErrSelect;
            K_star = kb.hi;
            J_star = kb.lo;
        } else {
            K_star = ~0ull;
            J_star = 0xFFFFFFFFu;
        }
        __syncthreads();
        const Pair96 kcut{K_star, J_star};
        each_s([&](u32 idx, u32 bits, u32 s) {
            if (is_member(idx, bits) &&
                (g.take_all || pair_le(sample_key(idx, seed), idx, kcut)))
                atomicAdd(&win_cnt[s], 1u);
        });
    }
    __syncthreads();

    // ---- output offset of every chunk: thread t holds the counters of chunks
    //      4*(1024*q + t) .. +3, q < kSlabs; prefix sums run slab after slab.
    //      This is the workgroup's first read of the counters, after the
    //      barrier that follows its atomics on them.
    u32 c[kSlabs][4], s4[kSlabs], inc[kSlabs];
#pragma unroll
    for (u32 q = 0; q < kSlabs; ++q) {
        const u32 s = 4u * (q * kFinThreads + tid);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (s < g.W) {
            if (__builtin_expect(wide, 0)) {
                // written by other workgroups of this grid: read where they were written
                v.x = __hip_atomic_load(&win_cnt[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v.y = __hip_atomic_load(&win_cnt[s + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v.z = __hip_atomic_load(&win_cnt[s + 2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v.w = __hip_atomic_load(&win_cnt[s + 3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                v = reinterpret_cast<const uint4 *>(win_cnt)[q * kFinThreads + tid];
            }
        }
        c[q][0] = v.x;
        c[q][1] = s + 1 < g.W ? v.y : 0u;
        c[q][2] = s + 2 < g.W ? v.z : 0u;
        c[q][3] = s + 3 < g.W ? v.w : 0u;
        s4[q] = c[q][0] + c[q][1] + c[q][2] + c[q][3];
    }
#pragma unroll
    for (u32 q = 0; q < kSlabs; ++q) inc[q] = wave_inclusive_sum(s4[q]);
    if (lane == kWave - 1) {
#pragma unroll
        for (u32 q = 0; q < kSlabs; ++q) scan32[q * kFinWaves + wave] = inc[q];
    }
    __syncthreads();
    {
        constexpr u32 n = kSlabs * kFinWaves;          // partial sums, a few per lane of wave 0
        constexpr u32 kEach = n / kWave;
        static_assert(n % kWave == 0 && kEach >= 1, "whole partial sums per lane");
        if (wave == 0) {
            u32 part[kEach], sum = 0;
#pragma unroll
            for (u32 j = 0; j < kEach; ++j) { part[j] = scan32[kEach * lane + j]; sum += part[j]; }
            const u32 xi = wave_inclusive_sum(sum);
            u32 running = xi - sum;
#pragma unroll
            for (u32 j = 0; j < kEach; ++j) { scan32[kEach * lane + j] = running; running += part[j]; }
            if (lane == kWave - 1) scan32[n] = xi;
        }
    }
    __syncthreads();
    const u64 total = scan32[kSlabs * kFinWaves];
#pragma unroll
    for (u32 q = 0; q < kSlabs; ++q) {
        const u32 s = 4u * (q * kFinThreads + tid);
        if (s < g.W) {
            uint4 o;
            o.x = scan32[q * kFinWaves + wave] + inc[q] - s4[q];
            o.y = o.x + c[q][0];
            o.z = o.y + c[q][1];
            o.w = o.z + c[q][2];
            reinterpret_cast<uint4 *>(chunk_base)[q * kFinThreads + tid] = o;
        }
    }
    if (total != g.k) err |= kErrCount;
    if (tid == 0) {
        ctl->err = err;
        ctl->path = path;
        ctl->T = T;
        ctl->I_star = I_star;
        ctl->K_star = K_star;
        ctl->J_star = J_star;
        ctl->n_b = n_bd;
        ctl->n_m = n_mm;
        ctl->W = g.W;
        ctl->U = g.U;
        ctl->UC = g.UC;
        ctl->count_greater = count_greater;
        ctl->ties = g.r - count_greater;
    }
}

// ---------------------------------------------------------------------------
// emit: members of the top-r set whose (key, index) is at or below the cut
// -> the message in index order; residual at the sent positions <- a - a.
// A winner's place is the output offset of its chunk plus the number of
// winners before it in the chunk; the latter is kept as the difference of two
// running totals over the wavefront's flat walk.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void
emit_body(Geom g, PhiloxSeed seed, const EncodeCtl *__restrict__ ctl,
       const u32 *__restrict__ seg_count, const uint2 *__restrict__ s_ent,
       const u32 *__restrict__ chunk_base,
       u32 *__restrict__ out_idx, float *__restrict__ out_val, float *residual)
{
    __shared__ uint2 row_queue[kWalkWaves][kRowQueue];
    const u32 u = blockIdx.x * kWalkWaves + threadIdx.x / kWave;
    if (u >= g.U) return;
    const u32 lane = lane_id();
    const Candidates cand{seg_count, s_ent, residual, g.d, g.C, g.U, g.UC, g.cap, ctl->dense != 0u};
    const UnitWalk walk(cand, u < g.U ? u : g.W, g.U, g.W);
    const u32 my_chunk = u + lane * g.U;
    const u32 my_base = (lane < g.UC && my_chunk < g.W) ? chunk_base[my_chunk] : 0u;
    const u32 T = ctl->T, I_star = ctl->I_star;
    const Pair96 kcut{ctl->K_star, ctl->J_star};
    const u64 below = lanes_below();
    u32 run = 0;          // winners at flat positions before this iteration
    u32 carry = 0;        // winners before the first entry of the chunk that runs into this iteration
    auto wins = [&](bool valid, u32 idx, u32 bits) {
        bool win = false;
        if (valid) {
            const u32 m = mag_of(bits);
            win = m > T || (m == T && idx <= I_star);
            if (win && !g.take_all) win = pair_le(sample_key(idx, seed), idx, kcut);
        }
        return win;
    };
    auto send = [&](u64 pos, u32 idx, u32 bits) {
        if (pos < g.k) {
            const float v = __uint_as_float(bits);
            out_idx[pos] = idx;
            out_val[pos] = v;
            residual[idx] = v - v;
        }
    };
    walk.for_each(cand, [&](bool valid, u32 i, u32 idx, u32 bits, u32 first, u32 p0) {
        const bool win = wins(valid, idx, bits);
        const u64 mask = __ballot(win);
        // winners before the first entry of this lane's chunk
        const u32 at_start =
            first >= p0 ? run + popc64(mask & ((1ull << (first - p0)) - 1ull)) : carry;
        const u32 base_c = __shfl(my_base, i, kWave);
        if (win) send((u64)base_c + (run + popc64(mask & below) - at_start), idx, bits);
        carry = __shfl(at_start, kWave - 1, kWave);
        run += popc64(mask);
    });
    // chunks read from the vector itself: what can be a member is gathered first,
    // then taken 64 at a time in index order; seen counts the chunk's winners so far
    u32 row_chunk = 0xFFFFFFFFu, seen = 0;
    if (__builtin_expect(walk.from_vector != 0ull, 0))
    walk.for_each_vector_entry(cand, row_queue[threadIdx.x / kWave],
                               [&](u32 bits) { return mag_of(bits) >= T; },
                               [&](bool valid, u32 i, u32 idx, u32 bits) {
        if (i != row_chunk) { row_chunk = i; seen = 0; }
        const bool win = wins(valid, idx, bits);
        const u64 mask = __ballot(win);
        if (mask == 0ull) return;
        const u32 base_c = __shfl(my_base, i, kWave);
        if (win) send((u64)base_c + seen + popc64(mask & below), idx, bits);
        seen += popc64(mask);
    });
}

// ---------------------------------------------------------------------------
// The kernels. One launch serves up to kMaxBatch independent vectors of the
// same sizes ("members": the workers of one node, or the tensors of one
// model): blockIdx.z is the member, and every member has its own workspace,
// ws_stride bytes after the previous one. Each member is computed exactly as
// if it were alone; batching only lets the short kernels of all members run
// side by side and the streaming kernel run on without draining in between.
// ---------------------------------------------------------------------------
constexpr u32 kMaxBatch = 16;

struct Batch {
    const float *grad[kMaxBatch];
    float *residual[kMaxBatch];
    u32 *out_idx[kMaxBatch];
    float *out_val[kMaxBatch];
    u32 seed_lo[kMaxBatch], seed_hi[kMaxBatch];
    u32 step_lo, step_hi;
    const u64 *step_dev;        // when not null, the step number is read from here instead
    char *ws;
    u64 ws_stride;
};

// what the workgroup's member works on
struct Member {
    const float *grad;
    float *residual;
    u32 *out_idx;
    float *out_val;
    PhiloxSeed seed;
    char *ws;
    __device__ __forceinline__ Member(const Batch &B)
    {
        const u32 i = blockIdx.z;
        grad = B.grad[i];
        residual = B.residual[i];
        out_idx = B.out_idx[i];
        out_val = B.out_val[i];
        u32 step_lo = B.step_lo, step_hi = B.step_hi;
        if (B.step_dev) {
            const u64 step = *B.step_dev;
            step_lo = (u32)step;
            step_hi = (u32)(step >> 32);
        }
        seed = PhiloxSeed{B.seed_lo[i], B.seed_hi[i], step_lo, step_hi};
        ws = B.ws + (u64)i * B.ws_stride;
    }
    template <class T>
    __device__ __forceinline__ T *at(u64 offset) const { return reinterpret_cast<T *>(ws + offset); }
};

__global__ void __launch_bounds__(kSampleThreads) k_sample(Batch B, Geom g, EncodeLayout L)
{
    const Member m(B);
    sample_body(m.grad, m.residual, g, m.seed, m.at<u32>(0), (u32)(L.zero_bytes / 4),
                m.at<u32>(L.samples));
}

__global__ void __launch_bounds__(kEstThreads) k_estimate(Batch B, Geom g, EncodeLayout L)
{
    const Member m(B);
    estimate_body(m.at<u32>(L.samples), g, m.at<EncodeCtl>(L.ctl));
}

template <bool kVec4, bool kAll>
__global__ void __launch_bounds__(kFusedThreads) k_fused(Batch B, Geom g, EncodeLayout L)
{
    const Member m(B);
    fused_body<kVec4, kAll>(m.grad, m.residual, g, m.seed, m.at<EncodeCtl>(L.ctl),
                            (u32)(L.zero_bytes / 4), m.at<u32>(L.partials), m.at<u32>(L.group_sums), m.at<u32>(L.seg_count),
                            m.at<uint2>(L.s_ent));
}

__global__ void __launch_bounds__(kPickThreads) k_pick(Batch B, u32 n_rows, Geom g, EncodeLayout L)
{
    const Member m(B);
    pick_body(m.at<u32>(L.partials), m.at<u32>(L.group_sums), n_rows, g, m.at<EncodeCtl>(L.ctl));
}

__global__ void __launch_bounds__(kWalkThreads) k_classify(Batch B, Geom g, EncodeLayout L)
{
    const Member m(B);
    classify_body(g, m.seed, m.at<EncodeCtl>(L.ctl), m.residual, m.at<u32>(L.seg_count),
                  m.at<uint2>(L.s_ent), m.at<u32>(L.win_cnt), m.at<u32>(L.bd_cnt),
                  m.at<u32>(L.blk_sure), m.at<u32>(L.n_m), m.at<u32>(L.n_b), m.at<u32>(L.blk_bmin),
                  m.at<u32>(L.blk_bmax), m.at<u64>(L.m_key), m.at<u32>(L.m_idx),
                  m.at<u32>(L.b_mag), m.at<u32>(L.b_idx));
}

__global__ void __launch_bounds__(kFinThreads) k_finalize(Batch B, Geom g, EncodeLayout L)
{
    const Member m(B);
    finalize_body(g, m.seed, m.at<EncodeCtl>(L.ctl), m.at<WideScratch>(L.wide), m.residual,
                  m.at<u32>(L.seg_count),
                  m.at<uint2>(L.s_ent), m.at<u32>(L.win_cnt), m.at<u32>(L.bd_cnt),
                  m.at<u32>(L.blk_sure), m.at<u32>(L.n_m), m.at<u32>(L.n_b),
                  m.at<u32>(L.blk_bmin), m.at<u32>(L.blk_bmax), m.at<u64>(L.m_key),
                  m.at<u32>(L.m_idx), m.at<u32>(L.b_mag), m.at<u32>(L.b_idx), m.at<u64>(L.dm_key),
                  m.at<u32>(L.dm_idx), m.at<u64>(L.db_key), m.at<u32>(L.db_idx),
                  m.at<u32>(L.chunk_base));
}

__global__ void __launch_bounds__(kWalkThreads) k_emit(Batch B, Geom g, EncodeLayout L)
{
    const Member m(B);
    emit_body(g, m.seed, m.at<EncodeCtl>(L.ctl), m.at<u32>(L.seg_count), m.at<uint2>(L.s_ent),
              m.at<u32>(L.chunk_base), m.out_idx, m.out_val, m.residual);
}

// ---------------------------------------------------------------------------
// Calibration (diagnostics): a = g + m into the residual buffer and nothing
// else, over the same chunks, with the same accesses and the same grid as
// the fused kernel: the speed of the bare read-read-write stream.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kFusedThreads)
k_stream_add(const float *__restrict__ grad, float *__restrict__ residual, u64 d, u32 C, u32 W)
{
    const u32 wave_stride = gridDim.x * kFusedWaves;
    for (u32 w = blockIdx.x * kFusedWaves + threadIdx.x / kWave; w < W; w += wave_stride) {
        const u64 c0 = (u64)w * C;
        const u64 c1 = c0 + C < d ? c0 + C : d;
        u64 base = c0;
        constexpr int NR = kFusedRows;
        for (; base + NR * kChunkQuantum <= c1; base += NR * kChunkQuantum) {
            const f32x4 *g4 = reinterpret_cast<const f32x4 *>(grad + base) + lane_id();
            f32x4 *m4 = reinterpret_cast<f32x4 *>(residual + base) + lane_id();
            f32x4 gv[NR], mv[NR];
#pragma unroll
            for (int u = 0; u < NR; ++u) {
                gv[u] = __builtin_nontemporal_load(g4 + u * kWave);
                mv[u] = __builtin_nontemporal_load(m4 + u * kWave);
            }
#pragma unroll
            for (int u = 0; u < NR; ++u) __builtin_nontemporal_store(gv[u] + mv[u], m4 + u * kWave);
        }
        for (u64 i = base + lane_id(); i < c1; i += kWave) residual[i] = grad[i] + residual[i];
    }
}

}  // namespace rtopk

// ===========================================================================
// C ABI
// ===========================================================================
using namespace rtopk;

static int check_sizes(uint64_t d, uint64_t r, uint64_t k)
{
    // domain of Definition 3, with 32-bit indices
    if (k < 1 || k > r || r > d || d > 0xFFFFFFFFull) return RTOPK_EINVAL;
    return RTOPK_OK;
}

extern "C" int rtopk_encode_workspace_bytes(uint64_t d, uint64_t r, uint64_t k, uint64_t *bytes)
{
    if (!bytes) return RTOPK_EINVAL;
    const int rc = check_sizes(d, r, k);
    if (rc) return rc;
    *bytes = make_layout(make_geom(d, r, k)).total;
    return RTOPK_OK;
}

namespace {
struct TraceRequest {
    int stage = 0;
    hipEvent_t begin = nullptr, end = nullptr;
};
thread_local TraceRequest g_trace;
thread_local unsigned g_force = 0;

// records the requested pair of events around one stage of the pipeline
struct StageScope {
    const TraceRequest &tr;
    hipStream_t stream;
    bool on;
    StageScope(const TraceRequest &t, int stage, hipStream_t s)
        : tr(t), stream(s), on(t.stage == stage)
    {
        if (on) (void)hipEventRecord(tr.begin, stream);
    }
    ~StageScope()
    {
        if (on) (void)hipEventRecord(tr.end, stream);
    }
};

// Workgroups of the streaming kernel: one per compute unit (all start
// together and share the chunks evenly, so none waits for a slot). Eight
// wavefronts per compute unit with 8 x 16 bytes in flight per lane saturate
// HBM; two or three workgroups per unit stream no faster, leave three times
// the histogram rows to add up and less room for kernels of other streams.
// The count of units is looked up at the first call on the device.
constexpr int kMaxDevices = 64;
constexpr int kFusedBlocksPerCU = 1;
// A batched launch holds several times that grid (one grid per member). Left
// to itself the device then keeps three workgroups of different members on
// every compute unit, and the interleaved streams cost 8% (443 instead of
// 407 us for eight vectors of 25.6 M elements). Each workgroup therefore also
// claims more than half of the unit's 160 KB of LDS, which it does not use: one
// workgroup per unit at any time, members streamed one after the other.
constexpr unsigned kFusedLdsClaim = 96u * 1024u;
std::mutex g_device_mutex;
unsigned g_fused_grid[kMaxDevices];

template <class K>
bool allow_lds_claim(K kernel)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)kFusedLdsClaim) == hipSuccess;
}

int fused_grid_limit(unsigned *out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RTOPK_EHIP;
    std::lock_guard<std::mutex> lock(g_device_mutex);
    if (g_fused_grid[dev] == 0) {
        int cus = 0, fit_t = 0, fit_f = 0;
        if (!allow_lds_claim(k_fused<true, false>) || !allow_lds_claim(k_fused<false, false>) ||
            !allow_lds_claim(k_fused<true, true>) || !allow_lds_claim(k_fused<false, true>))
            return RTOPK_EHIP;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&fit_t, k_fused<true, false>,
                                                         (int)kFusedThreads,
                                                         kFusedLdsClaim) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&fit_f, k_fused<false, true>,
                                                         (int)kFusedThreads,
                                                         kFusedLdsClaim) != hipSuccess)
            return RTOPK_EHIP;
        int per_cu = fit_t < fit_f ? fit_t : fit_f;
        per_cu = per_cu < kFusedBlocksPerCU ? per_cu : kFusedBlocksPerCU;
        if (cus < 1 || per_cu < 1) return RTOPK_EHIP;
        const unsigned grid = (unsigned)cus * (unsigned)per_cu;
        g_fused_grid[dev] = grid > kMaxFusedBlocks ? kMaxFusedBlocks : grid;
    }
    *out = g_fused_grid[dev];
    return RTOPK_OK;
}
}  // namespace

extern "C" int rtopk_force_next_encode(unsigned flags)
{
    if (flags & ~(unsigned)(RTOPK_FORCE_ESTIMATE_MISS | RTOPK_FORCE_KEY_WINDOW_MISS |
                            RTOPK_FORCE_CHECK_IN_ABORT | RTOPK_FORCE_BRACKET_LOW |
                            RTOPK_FORCE_BARRIER_TIMEOUT))
        return RTOPK_EINVAL;
    g_force = flags;
    return RTOPK_OK;
}

extern "C" int rtopk_trace_next_encode(int stage, void *ev_begin, void *ev_end)
{
    if (stage != 0 && (!ev_begin || !ev_end)) return RTOPK_EINVAL;
    g_trace.stage = stage;
    g_trace.begin = (hipEvent_t)ev_begin;
    g_trace.end = (hipEvent_t)ev_end;
    return RTOPK_OK;
}

#define RTOPK_LAUNCH_CHECK()                              \
    do {                                                  \
        if (hipGetLastError() != hipSuccess) return RTOPK_EHIP; \
    } while (0)

static int encode_batch_impl(uint32_t n, const float *const *grad, float *const *residual,
                             uint64_t d, uint64_t r, uint64_t k, const uint64_t *seed,
                             uint64_t step, const uint64_t *step_dev, uint32_t *const *out_idx,
                             float *const *out_val, void *workspace, uint64_t workspace_bytes,
                             void *stream_v)
{
    if (n < 1 || !grad || !residual || !seed || !out_idx || !out_val) return RTOPK_EINVAL;
    const int rc = check_sizes(d, r, k);
    if (rc) return rc;
    bool vec4 = true;
    for (uint32_t i = 0; i < n; ++i) {
        if (!grad[i] || !residual[i] || !out_idx[i] || !out_val[i]) return RTOPK_EINVAL;
        const uintptr_t g0 = (uintptr_t)grad[i], m0 = (uintptr_t)residual[i];
        if (g0 < m0 + d * 4 && m0 < g0 + d * 4) return RTOPK_EINVAL;
        vec4 = vec4 && ((g0 | m0) & 15u) == 0;
    }
    Geom g = make_geom(d, r, k);
    const EncodeLayout L = make_layout(g);
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes / n < L.total)
        return RTOPK_EWORKSPACE;
    const unsigned force = g_force;
    g_force = 0;
    // a forced estimate miss belongs to the general path; a forced window miss is
    // honoured on the r == d path too (it then walks the vector itself)
    if (force & RTOPK_FORCE_ESTIMATE_MISS) g.all_members = 0u;
    if (force & RTOPK_FORCE_ESTIMATE_MISS) g.force_dense = 1u;
    if (force & RTOPK_FORCE_CHECK_IN_ABORT) g.force_abort = 1u;
    if (force & RTOPK_FORCE_BRACKET_LOW) g.force_low = 1u;
    if (force & RTOPK_FORCE_BARRIER_TIMEOUT) g.force_timeout = 1u;
    if ((force & RTOPK_FORCE_KEY_WINDOW_MISS) && !g.take_all) {
        g.K_lo = g.K_hi = 0;       // a window that holds no key: the exact selection must run
        g.k_nlz = 63u;
    }
    hipStream_t stream = (hipStream_t)stream_v;
    unsigned grid_limit = 0;
    const int rc2 = fused_grid_limit(&grid_limit);
    if (rc2) return rc2;
    unsigned fgrid = (g.W + kFusedWaves - 1) / kFusedWaves;
    if (fgrid > grid_limit) fgrid = grid_limit;

    const TraceRequest trace = g_trace;
    g_trace = TraceRequest{};
    StageScope whole(trace, RTOPK_STAGE_ALL, stream);

    for (uint32_t first = 0; first < n; first += kMaxBatch) {
        const unsigned nb = n - first < kMaxBatch ? n - first : kMaxBatch;
        Geom gg = g;                    // this launch group's share-out of the walking kernels
        set_units(gg, nb);
        Batch B{};
        for (unsigned i = 0; i < nb; ++i) {
            B.grad[i] = grad[first + i];
            B.residual[i] = residual[first + i];
            B.out_idx[i] = out_idx[first + i];
            B.out_val[i] = out_val[first + i];
            B.seed_lo[i] = (u32)seed[first + i];
            B.seed_hi[i] = (u32)(seed[first + i] >> 32);
        }
        B.step_lo = (u32)step;
        B.step_hi = (u32)(step >> 32);
        B.step_dev = step_dev;
        B.ws = (char *)workspace + (u64)first * L.total;
        B.ws_stride = L.total;
        const dim3 fg(fgrid, 1, nb);
        if (g.all_members) {
            // r == d (random-k): no estimate, no histogram, no threshold
            StageScope sc(trace, RTOPK_STAGE_FUSED, stream);
            if (vec4)
                k_fused<true, true><<<fg, kFusedThreads, kFusedLdsClaim, stream>>>(B, gg, L);
            else
                k_fused<false, true><<<fg, kFusedThreads, kFusedLdsClaim, stream>>>(B, gg, L);
            RTOPK_LAUNCH_CHECK();
        } else {
            {
                StageScope sc(trace, RTOPK_STAGE_PREPARE, stream);
                k_sample<<<dim3(kSampleLoc / kSampleThreads, 1, nb), kSampleThreads, 0, stream>>>(
                    B, gg, L);
                RTOPK_LAUNCH_CHECK();
                k_estimate<<<dim3(1, 1, nb), kEstThreads, 0, stream>>>(B, gg, L);
                RTOPK_LAUNCH_CHECK();
            }
            {
                StageScope sc(trace, RTOPK_STAGE_FUSED, stream);
                if (vec4)
                    k_fused<true, false><<<fg, kFusedThreads, kFusedLdsClaim, stream>>>(B, gg, L);
                else
                    k_fused<false, false><<<fg, kFusedThreads, kFusedLdsClaim, stream>>>(B, gg, L);
                RTOPK_LAUNCH_CHECK();
            }
        }
        {
            StageScope sc(trace, RTOPK_STAGE_CLASSIFY, stream);
            if (!g.all_members) {
                k_pick<<<dim3(1, 1, nb), kPickThreads, 0, stream>>>(B, fgrid, gg, L);
                RTOPK_LAUNCH_CHECK();
            }
            k_classify<<<dim3(gg.G3, 1, nb), kWalkThreads, 0, stream>>>(B, gg, L);
            RTOPK_LAUNCH_CHECK();
        }
        {
            StageScope sc(trace, RTOPK_STAGE_FINALIZE, stream);
            // long vectors: enough workgroups for the exact fallback over all candidates
            // (all but the first leave at once when the short lists decide)
            // (the kernel's workgroups are resident one per compute unit: a batch shares them)
            unsigned fin_grid = 1u;
            if (g.W >= kWideMinChunks) {
                fin_grid = 256u / nb;
                fin_grid = fin_grid > kWideBlocks ? kWideBlocks : (fin_grid < 16u ? 16u : fin_grid);
            }
            k_finalize<<<dim3(fin_grid, 1, nb), kFinThreads, 0, stream>>>(B, gg, L);
            RTOPK_LAUNCH_CHECK();
        }
        {
            StageScope sc(trace, RTOPK_STAGE_EMIT, stream);
            k_emit<<<dim3(gg.G3, 1, nb), kWalkThreads, 0, stream>>>(B, gg, L);
            RTOPK_LAUNCH_CHECK();
        }
    }
    return RTOPK_OK;
}

extern "C" int rtopk_encode_batch(uint32_t n, const float *const *grad, float *const *residual,
                                  uint64_t d, uint64_t r, uint64_t k, const uint64_t *seed,
                                  uint64_t step, uint32_t *const *out_idx, float *const *out_val,
                                  void *workspace, uint64_t workspace_bytes, void *stream_v)
{
    return encode_batch_impl(n, grad, residual, d, r, k, seed, step, nullptr, out_idx, out_val,
                             workspace, workspace_bytes, stream_v);
}

extern "C" int rtopk_encode_batch_device_step(uint32_t n, const float *const *grad,
                                              float *const *residual, uint64_t d, uint64_t r,
                                              uint64_t k, const uint64_t *seed,
                                              const uint64_t *step_device,
                                              uint32_t *const *out_idx, float *const *out_val,
                                              void *workspace, uint64_t workspace_bytes,
                                              void *stream_v)
{
    if (!step_device || ((uintptr_t)step_device & 7u)) return RTOPK_EINVAL;
    return encode_batch_impl(n, grad, residual, d, r, k, seed, 0, step_device, out_idx, out_val,
                             workspace, workspace_bytes, stream_v);
}

extern "C" int rtopk_encode(const float *grad, float *residual, uint64_t d, uint64_t r,
                            uint64_t k, uint64_t seed, uint64_t step, uint32_t *out_idx,
                            float *out_val, void *workspace, uint64_t workspace_bytes,
                            void *stream_v)
{
    return rtopk_encode_batch(1, &grad, &residual, d, r, k, &seed, step, &out_idx, &out_val,
                              workspace, workspace_bytes, stream_v);
}

extern "C" int rtopk_diag_stream_add(const float *grad, float *residual, uint64_t d,
                                     void *stream_v)
{
    if (!grad || !residual || d < 1 || d > 0xFFFFFFFFull) return RTOPK_EINVAL;
    const uintptr_t g0 = (uintptr_t)grad, m0 = (uintptr_t)residual;
    if (((g0 | m0) & 15u) || (g0 < m0 + d * 4 && m0 < g0 + d * 4)) return RTOPK_EINVAL;
    const Geom g = make_geom(d, d, d);                     // the chunking only
    unsigned grid_limit = 0;
    const int rc = fused_grid_limit(&grid_limit);
    if (rc) return rc;
    unsigned fgrid = (g.W + kFusedWaves - 1) / kFusedWaves;
    if (fgrid > grid_limit) fgrid = grid_limit;
    k_stream_add<<<fgrid, kFusedThreads, 0, (hipStream_t)stream_v>>>(grad, residual, d, g.C, g.W);
    RTOPK_LAUNCH_CHECK();
    return RTOPK_OK;
}

extern "C" int rtopk_encode_stats(const void *workspace, void *stream_v,
                                  rtopk_encode_stats_t *host_out)
{
    if (!workspace || !host_out) return RTOPK_EINVAL;
    hipStream_t stream = (hipStream_t)stream_v;
    if (hipStreamSynchronize(stream) != hipSuccess) return RTOPK_EHIP;
    EncodeCtl c;
    if (hipMemcpy(&c, workspace, sizeof c, hipMemcpyDeviceToHost) != hipSuccess)
        return RTOPK_EHIP;
    // candidates kept by the streaming kernel: the chunk sizes, added up here
    uint64_t superset = 0;
    if (c.W > 0 && c.W <= kTargetChunks && c.U > 0 && c.UC > 0 && (u64)c.U * c.UC <= kTargetChunks &&
        c.W <= c.U * c.UC) {
        const EncodeLayout L = make_layout(Geom{});   // the offset of seg_count is fixed
        std::vector<u32> counts(kTargetChunks);
        if (hipMemcpy(counts.data(), (const char *)workspace + L.seg_count,
                      (size_t)kTargetChunks * 4, hipMemcpyDeviceToHost) != hipSuccess)
            return RTOPK_EHIP;
        for (u32 s2 = 0; s2 < c.W; ++s2) superset += counts[chunk_slot(s2, c.U, c.UC)];
    }
    host_out->error_flags = c.err;
    host_out->path = c.path | (c.dense ? 2u : 0u);
    host_out->threshold_bits = c.T;
    host_out->boundary_list_size = c.n_b;
    host_out->count_greater = c.count_greater;
    host_out->ties_taken = c.ties;
    host_out->superset_size = superset;
    host_out->key_list_size = c.n_m;
    return RTOPK_OK;
}
