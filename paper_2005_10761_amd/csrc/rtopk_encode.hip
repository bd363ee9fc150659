// rtopk_encode: one node-side step of Algorithm 1 (error compensation, the
// rTop-k operator of Definition 3, residual write-back) as a chain of gfx950
// kernels. All cross-kernel state lives in the caller's workspace.
//
// The vector is cut into W contiguous chunks, one per wavefront, and every
// chunk owns a slice of the candidate buffer S as long as the chunk itself.
// A wavefront that streams its chunk appends the entries it keeps to its own
// slice in index order and finally stores how many it kept. S is therefore
// ordered by index without any cross-workgroup scan, ticket or fence, and a
// slice can never overflow. Later kernels walk S chunk by chunk.
//
// Pipeline:
//   init       zero the control block and the two global histograms
//   fused      a = g + m, stored into the residual buffer; histogram of the
//              top 12 magnitude bits (12d bytes, the dominant kernel)
//   scan       every workgroup picks the bucket b1 that holds the r-th largest
//              magnitude; entries in bucket b1 or above -> S; 4096-bin
//              histogram of the next 12 bits of the bucket-b1 entries (4d)
//   classify   every workgroup picks the deciding level-2 bin. Entries of S
//              above it are certain members of the top-r set: their Philox
//              key is compared with an a-priori window [K_lo, K_hi] around
//              the k-th smallest of r uniform keys - below: certain winner
//              (counted per unit), inside: copied to the short list M.
//              Entries inside the deciding bin are copied to the short list B
//   finalize   one workgroup: exact r-th largest (magnitude, lower index
//              first) inside B -> (T, I*); members of B join the key lists;
//              exact (k - #certain)-th smallest (key, index) in M -> (K*, J*);
//              prefix sum of the winners per unit. Whenever a short list
//              overflowed or the key window missed, the same quantities are
//              found by radix selection over all of S instead (slow, exact)
//   emit       entries of S that are members and winners -> the message in
//              index order, starting at the unit's prefix; residual at the
//              sent positions <- a - a
//
// What the hardware punishes shaped this: a device-scope fence inside a
// kernel costs tens of microseconds once a few hundred workgroups execute
// one, and atomics on a single address retire at about one per 12 ns. So no
// kernel here uses a fence, a ticket or a "last workgroup out" protocol;
// workgroups never wait for each other; global atomics only go to histogram
// bins; small decisions are recomputed by every workgroup that needs them.
#include "rtopk_common.h"
#include "../../include/rtopk.h"

#include <math.h>

namespace rtopk {

constexpr int kShift1 = 19;                   // level 1: top 12 of the 31 magnitude bits
constexpr int kBins1 = 1 << 12;
constexpr int kBins2 = 1 << 12;               // level 2: next 12 bits of the picked bucket
constexpr int kShift2 = kShift1 - 12;

constexpr u32 kChunkQuantum = 256;            // one wavefront iteration: 64 lanes x 4 elements
constexpr u32 kTargetChunks = 8192;
constexpr u32 kMaxUnits = 4096;               // a unit = the chunks one wavefront of classify/emit walks
constexpr u32 kWalkThreads = 256;             // classify / emit / scan workgroups: 4 wavefronts
constexpr u32 kWalkWaves = kWalkThreads / kWave;
constexpr u32 kMaxWalkBlocks = kMaxUnits / kWalkWaves;
constexpr u32 kListCap = 512;                 // short-list slots per classify workgroup
constexpr int kFinThreads = 1024;
constexpr u32 kStageB = 512, kStageM = 2560;  // short lists that fit are selected in LDS

constexpr u32 kErrSelect = 2u;                // a selection found no element of the requested rank
constexpr u32 kErrCount = 4u;                 // the winners did not add up to k

struct EncodeCtl {
    u32 err;
    u32 path;           // 0: short lists; 1: some quantity came from selection over all of S
    // written by workgroup 0 of k_scan
    u32 h_lo;           // lowest magnitude pattern covered by the level-2 histogram
    u32 h_shift;        // log2 of the patterns per level-2 bin
    u64 c_above;        // entries above the level-2 range
    // written by workgroup 0 of k_classify
    u32 bd_lo, bd_hi;   // pattern range of the deciding level-2 bin
    u64 c_def;          // entries above bd_hi
    u32 overflow;       // a short-list region of some classify workgroup was full
    u32 pad0;
    // written by k_finalize
    u32 T, I_star;      // last member of the top-r set in (magnitude desc, index asc) order
    u64 K_star;         // last winner in (key asc, index asc) order
    u32 J_star;
    u32 n_b, n_m, pad1;
    u64 superset, count_greater, ties;
};

// Geometry and sampling window: a pure function of (d, r, k), computed on the host.
struct Geom {
    u64 d, r, k;
    u32 C;              // elements per chunk (multiple of 256)
    u32 W;              // chunks
    u32 SU;             // chunks per unit
    u32 U;              // units
    u32 G3;             // classify / emit workgroups
    u32 take_all;       // k == r: every member is sent, keys are never looked at
    u64 K_lo, K_hi;     // key window
    u32 k_nlz;          // leading zeros of K_hi - K_lo
    u32 pad;
};

struct EncodeLayout {
    u64 ctl, hist1, hist2, zero_bytes;
    u64 seg_count, win_sure, unit_base, n_m, n_b;
    u64 m_key, m_idx, b_mag, b_idx;
    u64 dm_key, dm_idx, db_key, db_idx;
    u64 s_idx, s_val;
    u64 total;
};

static Geom make_geom(u64 d, u64 r, u64 k)
{
    Geom g{};
    g.d = d; g.r = r; g.k = k;
    u64 per = (d + kTargetChunks - 1) / kTargetChunks;
    per = (per + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    g.C = (u32)per;
    g.W = (u32)((d + per - 1) / per);
    g.SU = (g.W + kMaxUnits - 1) / kMaxUnits;
    g.U = (g.W + g.SU - 1) / g.SU;
    g.G3 = (g.U + kWalkWaves - 1) / kWalkWaves;
    g.take_all = (k == r) ? 1u : 0u;
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

static EncodeLayout make_layout(const Geom &g)
{
    EncodeLayout L{};
    u64 o = 0;
    auto take = [&](u64 bytes) { u64 at = o; o = align_up(o + bytes, 256); return at; };
    L.ctl = take(sizeof(EncodeCtl));
    L.hist1 = take(kBins1 * 4);
    L.hist2 = take(kBins2 * 4);
    L.zero_bytes = o;
    L.seg_count = take((u64)g.W * 4);
    L.win_sure = take((u64)g.U * 4);
    L.unit_base = take((u64)g.U * 4);
    L.n_m = take((u64)g.G3 * 4);
    L.n_b = take((u64)g.G3 * 4);
    const u64 slots = (u64)g.G3 * kListCap;
    L.m_key = take(slots * 8);
    L.m_idx = take(slots * 4);
    L.b_mag = take(slots * 4);
    L.b_idx = take(slots * 4);
    L.dm_key = take(2 * slots * 8);
    L.dm_idx = take(2 * slots * 4);
    L.db_key = take(slots * 8);
    L.db_idx = take(slots * 4);
    const u64 cap = (u64)g.W * g.C;
    L.s_idx = take(cap * 4);
    L.s_val = take(cap * 4);
    L.total = o;
    return L;
}

__device__ __forceinline__ u32 mag_of(u32 bits) { return bits & 0x7FFFFFFFu; }
__device__ __forceinline__ u32 popc64(u64 m) { return (u32)__popcll((unsigned long long)m); }

// ---------------------------------------------------------------------------
// workgroup-wide sums of one u64 per thread (thread order)
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 block_exclusive_sum(u64 v, u64 *lds /* >= waves + 1 words */)
{
    const u32 lane = lane_id(), wave = threadIdx.x / kWave, nw = blockDim.x / kWave;
    u64 inc = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const u64 t = __shfl_up(inc, off, kWave);
        if (lane >= (u32)off) inc += t;
    }
    if (lane == kWave - 1) lds[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 run = 0;
        for (u32 w = 0; w < nw; ++w) { const u64 t = lds[w]; lds[w] = run; run += t; }
        lds[nw] = run;
    }
    __syncthreads();
    const u64 res = lds[wave] + inc - v;
    __syncthreads();
    return res;
}

__device__ __forceinline__ u64 block_sum(u64 v, u64 *lds /* >= waves + 1 words */)
{
    const u32 nw = blockDim.x / kWave;
    v = wave_sum_u64(v);
    if (lane_id() == 0) lds[threadIdx.x / kWave] = v;
    __syncthreads();
    u64 total = 0;
    for (u32 w = 0; w < nw; ++w) total += lds[w];
    __syncthreads();
    return total;
}

// Whole workgroup: walking the bins from the top, find the bin b with
// #(bins above b) < need <= #(bins >= b). Stores b and the population above
// it; the caller synchronises before reading them.
__device__ __forceinline__ void block_pick_desc(const u32 *hist, int nbins, u64 need,
                                                u32 *out_bin, u64 *out_before, u64 *lds)
{
    const int per = (nbins + (int)blockDim.x - 1) / (int)blockDim.x;
    const int first = (int)threadIdx.x * per;      // position in walking order
    u64 mine = 0;
    for (int q = 0; q < per; ++q) {
        const int pos = first + q;
        if (pos < nbins) mine += hist[nbins - 1 - pos];
    }
    const u64 before = block_exclusive_sum(mine, lds);
    if (before < need && need <= before + mine) {
        u64 run = before;
        for (int q = 0; q < per; ++q) {
            const int pos = first + q;
            if (pos >= nbins) break;
            const int bin = nbins - 1 - pos;
            const u64 h = hist[bin];
            if (run + h >= need) { *out_bin = (u32)bin; *out_before = run; break; }
            run += h;
        }
    }
}

// ---------------------------------------------------------------------------
// init: clear what the later kernels accumulate into
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_init(u32 *zero_base, u32 words)
{
    for (u32 i = blockIdx.x * blockDim.x + threadIdx.x; i < words; i += gridDim.x * blockDim.x)
        zero_base[i] = 0u;
}

// ---------------------------------------------------------------------------
// fused residual add + level-1 histogram (12d bytes of HBM traffic)
// ---------------------------------------------------------------------------
constexpr int kFusedThreads = 1024;
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool kVec4>
__global__ void __launch_bounds__(kFusedThreads)
k_fused_add_hist(const float *__restrict__ grad, float *__restrict__ residual, u64 d, u32 *hist1)
{
    __shared__ u32 h[kBins1];
    for (int b = threadIdx.x; b < kBins1; b += kFusedThreads) h[b] = 0u;
    __syncthreads();

    if (kVec4) {
        const u64 nvec = d / 4;
        const f32x4 *g4 = reinterpret_cast<const f32x4 *>(grad);
        f32x4 *m4 = reinterpret_cast<f32x4 *>(residual);
        const u64 stride = (u64)gridDim.x * kFusedThreads;
        u64 v = (u64)blockIdx.x * kFusedThreads + threadIdx.x;
        auto body = [&](const f32x4 &g, const f32x4 &m, u64 at) {
            const f32x4 a = g + m;
            m4[at] = a;
            const u32 d0 = mag_of(__float_as_uint(a.x)) >> kShift1,
                      d1 = mag_of(__float_as_uint(a.y)) >> kShift1,
                      d2 = mag_of(__float_as_uint(a.z)) >> kShift1,
                      d3 = mag_of(__float_as_uint(a.w)) >> kShift1;
            // runs of equal digits (zero rows, constant blocks): one add per wave
            const u32 lead = __builtin_amdgcn_readfirstlane(d0);
            const bool same = (d0 == lead) & (d1 == lead) & (d2 == lead) & (d3 == lead);
            const u64 active = __ballot(true);
            if (__ballot(same) == active) {
                if (lane_id() == (u32)(__ffsll((unsigned long long)active) - 1))
                    atomicAdd(&h[lead], 4u * popc64(active));
            } else {
                atomicAdd(&h[d0], 1u); atomicAdd(&h[d1], 1u);
                atomicAdd(&h[d2], 1u); atomicAdd(&h[d3], 1u);
            }
        };
        for (; v + 3 * stride < nvec; v += 4 * stride) {
            f32x4 g[4], m[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                g[u] = __builtin_nontemporal_load(&g4[v + u * stride]);
                m[u] = m4[v + u * stride];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) body(g[u], m[u], v + u * stride);
        }
        for (; v < nvec; v += stride) {
            const f32x4 g = __builtin_nontemporal_load(&g4[v]);
            const f32x4 m = m4[v];
            body(g, m, v);
        }
        if (blockIdx.x == 0 && threadIdx.x < (d & 3)) {
            const u64 i = nvec * 4 + threadIdx.x;
            const float a = grad[i] + residual[i];
            residual[i] = a;
            atomicAdd(&h[mag_of(__float_as_uint(a)) >> kShift1], 1u);
        }
    } else {
        const u64 stride = (u64)gridDim.x * kFusedThreads;
        for (u64 i = (u64)blockIdx.x * kFusedThreads + threadIdx.x; i < d; i += stride) {
            const float a = grad[i] + residual[i];
            residual[i] = a;
            atomicAdd(&h[mag_of(__float_as_uint(a)) >> kShift1], 1u);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins1; b += kFusedThreads) {
        const u32 c = h[b];
        if (c) atomicAdd(&hist1[b], c);
    }
}

// ---------------------------------------------------------------------------
// One wavefront iteration of a chunk scan: 256 consecutive elements starting
// at `base`, of which those below `end` exist. Layout of the four elements a
// lane holds: kVec4 -> base + 4*lane + e (one 16-byte load); otherwise
// base + 64*e + lane (four coalesced 4-byte loads, any alignment).
// Kept entries are appended to the wavefront's slice in index order.
// ---------------------------------------------------------------------------
template <bool kVec4>
__device__ __forceinline__ u64 elem_index(u64 base, int e)
{
    return kVec4 ? base + 4ull * lane_id() + (u64)e : base + 64ull * (u64)e + lane_id();
}

template <bool kVec4>
__device__ __forceinline__ void load_row(const float *__restrict__ a, u64 base, u64 end,
                                         u32 (&bits)[4], bool (&valid)[4])
{
    if (kVec4) {
        const u64 i0 = base + 4ull * lane_id();
        if (i0 + 3 < end) {
            const float4 v = *reinterpret_cast<const float4 *>(a + i0);
            bits[0] = __float_as_uint(v.x); bits[1] = __float_as_uint(v.y);
            bits[2] = __float_as_uint(v.z); bits[3] = __float_as_uint(v.w);
            valid[0] = valid[1] = valid[2] = valid[3] = true;
            return;
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const u64 i = elem_index<kVec4>(base, e);
        valid[e] = i < end;
        bits[e] = valid[e] ? __float_as_uint(a[i]) : 0u;
    }
}

template <bool kVec4>
__device__ __forceinline__ void append_hits(const u32 (&bits)[4], const bool (&hit)[4], u64 base,
                                            u32 &run, u32 *__restrict__ my_idx,
                                            u32 *__restrict__ my_val)
{
    const u64 b0 = __ballot(hit[0]), b1 = __ballot(hit[1]), b2 = __ballot(hit[2]),
              b3 = __ballot(hit[3]);
    if ((b0 | b1 | b2 | b3) == 0ull) return;
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
        if (hit[e]) {
            my_idx[pos[e]] = (u32)elem_index<kVec4>(base, e);
            my_val[pos[e]] = bits[e];
        }
    }
    run += popc64(b0) + popc64(b1) + popc64(b2) + popc64(b3);
}

// ---------------------------------------------------------------------------
// scan: entries whose level-1 digit is at or above the picked bucket -> S;
// level-2 histogram of the entries inside the bucket. Reads a once (4d).
// ---------------------------------------------------------------------------
template <bool kVec4>
__global__ void __launch_bounds__(kWalkThreads)
k_scan(const float *__restrict__ a, Geom g, EncodeCtl *ctl, const u32 *__restrict__ hist1,
       u32 *hist2, u32 *__restrict__ seg_count, u32 *__restrict__ s_idx,
       u32 *__restrict__ s_val)
{
    __shared__ u32 h2[kBins2];
    __shared__ u64 scan_lds[kWalkWaves + 1];
    __shared__ u32 bin_s;
    __shared__ u64 before_s;
    for (int b = threadIdx.x; b < kBins2; b += kWalkThreads) h2[b] = 0u;
    block_pick_desc(hist1, kBins1, g.r, &bin_s, &before_s, scan_lds);
    __syncthreads();
    const u32 t_lo = bin_s << kShift1;
    const u32 h_hi = t_lo | ((1u << kShift1) - 1u);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ctl->h_lo = t_lo;
        ctl->h_shift = kShift2;
        ctl->c_above = before_s;
    }

    const u32 w = blockIdx.x * kWalkWaves + threadIdx.x / kWave;
    if (w < g.W) {
        const u64 c0 = (u64)w * g.C;
        const u64 c1 = c0 + g.C < g.d ? c0 + g.C : g.d;
        u32 *my_idx = s_idx + c0, *my_val = s_val + c0;
        u32 run = 0;
        auto process = [&](const u32 (&bits)[4], const bool (&valid)[4], u64 base) {
            bool hit[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const u32 m = mag_of(bits[e]);
                hit[e] = valid[e] && m >= t_lo;
                if (hit[e] && m <= h_hi) atomicAdd(&h2[(m - t_lo) >> kShift2], 1u);
            }
            append_hits<kVec4>(bits, hit, base, run, my_idx, my_val);
        };
        u64 base = c0;
        for (; base + 4 * kChunkQuantum <= c1; base += 4 * kChunkQuantum) {
            u32 bits[4][4];
            bool valid[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                load_row<kVec4>(a, base + u * kChunkQuantum, c1, bits[u], valid[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) process(bits[u], valid[u], base + u * kChunkQuantum);
        }
        for (; base < c1; base += kChunkQuantum) {
            u32 bits[4];
            bool valid[4];
            load_row<kVec4>(a, base, c1, bits, valid);
            process(bits, valid, base);
        }
        if (lane_id() == 0) seg_count[w] = run;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins2; b += kWalkThreads) {
        const u32 c = h2[b];
        if (c) atomicAdd(&hist2[b], c);
    }
}

// ---------------------------------------------------------------------------
// classify: walk S; certain members are keyed against the window, entries
// of the deciding level-2 bin go to the short list B.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kWalkThreads)
k_classify(Geom g, PhiloxSeed seed, EncodeCtl *ctl, const u32 *__restrict__ hist2,
           const u32 *__restrict__ seg_count, const u32 *__restrict__ s_idx,
           const u32 *__restrict__ s_val, u32 *__restrict__ win_sure, u32 *__restrict__ n_m,
           u32 *__restrict__ n_b, u64 *__restrict__ m_key, u32 *__restrict__ m_idx,
           u32 *__restrict__ b_mag, u32 *__restrict__ b_idx)
{
    __shared__ u64 scan_lds[kWalkWaves + 1];
    __shared__ u32 bin_s, cnt_m, cnt_b;
    __shared__ u64 before_s;
    if (threadIdx.x == 0) { cnt_m = 0u; cnt_b = 0u; }
    const u64 c_above = ctl->c_above;
    const u32 h_lo = ctl->h_lo, h_shift = ctl->h_shift;
    block_pick_desc(hist2, kBins2, g.r - c_above, &bin_s, &before_s, scan_lds);
    __syncthreads();
    const u32 bd_lo = h_lo + (bin_s << h_shift);
    const u32 bd_hi = bd_lo + ((1u << h_shift) - 1u);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ctl->bd_lo = bd_lo;
        ctl->bd_hi = bd_hi;
        ctl->c_def = c_above + before_s;
    }

    const u32 u = blockIdx.x * kWalkWaves + threadIdx.x / kWave;
    const u32 lane = lane_id();
    const u64 slot0 = (u64)blockIdx.x * kListCap;
    if (u < g.U) {
        u32 sure = 0;
        const u32 s_end = (u + 1) * g.SU < g.W ? (u + 1) * g.SU : g.W;
        for (u32 s = u * g.SU; s < s_end; ++s) {
            const u32 n = seg_count[s];
            const u64 at = (u64)s * g.C;
            for (u32 j = lane; j < n; j += kWave) {
                const u32 idx = s_idx[at + j];
                const u32 m = mag_of(s_val[at + j]);
                if (m > bd_hi) {
                    if (g.take_all) { ++sure; continue; }
                    const u64 key = sample_key(idx, seed);
                    if (key < g.K_lo) {
                        ++sure;
                    } else if (key <= g.K_hi) {
                        const u32 p = atomicAdd(&cnt_m, 1u);
                        if (p < kListCap) { m_key[slot0 + p] = key; m_idx[slot0 + p] = idx; }
                    }
                } else if (m >= bd_lo) {
                    const u32 p = atomicAdd(&cnt_b, 1u);
                    if (p < kListCap) { b_mag[slot0 + p] = m; b_idx[slot0 + p] = idx; }
                }
            }
        }
        sure = (u32)wave_sum_u64(sure);
        if (lane == 0) win_sure[u] = sure;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        n_m[blockIdx.x] = cnt_m < kListCap ? cnt_m : kListCap;
        n_b[blockIdx.x] = cnt_b < kListCap ? cnt_b : kListCap;
        if (cnt_m > kListCap || cnt_b > kListCap) ctl->overflow = 1u;
    }
}

// ---------------------------------------------------------------------------
// Radix selection, most significant byte first, over distinct 96-bit strings
// hi:lo (hi 64 bits, lo 32 bits). for_each(f) calls f(hi, lo) for every
// element this thread is responsible for (the elements are split over the
// workgroup in a way that does not change between calls). Returns the
// rank-th smallest string (rank is 1-based). Bytes before first_byte are
// known to be zero in every string. *ok is cleared when fewer than `rank`
// strings exist.
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
                                                 u32 *h /* 256 */, u64 *scratch /* 4 */, bool *ok)
{
    u64 phi = 0;
    u32 plo = 0;
    u64 need = rank;
    int j = first_byte;
    *ok = true;
    for (; j < 12; ++j) {
        for (u32 b = threadIdx.x; b < 256u; b += blockDim.x) h[b] = 0u;
        if (threadIdx.x == 0) { scratch[0] = 0; scratch[1] = 0; scratch[2] = 0; }
        __syncthreads();
        for_each([&](u64 hi, u32 lo) {
            if (pair_matches(hi, lo, phi, plo, j)) atomicAdd(&h[pair_byte(hi, lo, j)], 1u);
        });
        __syncthreads();
        if (threadIdx.x < (u32)kWave) {
            const u32 lane = threadIdx.x;
            u64 c[4], mine = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { c[q] = h[4 * lane + q]; mine += c[q]; }
            u64 inc = mine;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const u64 t = __shfl_up(inc, off, kWave);
                if (lane >= (u32)off) inc += t;
            }
            u64 run = inc - mine;
            if (run < need && need <= inc) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (run < need && need <= run + c[q]) {
                        scratch[0] = 4 * lane + q; scratch[1] = run; scratch[2] = c[q];
                    }
                    run += c[q];
                }
            }
        }
        __syncthreads();
        const u32 bin = (u32)scratch[0];
        const u64 in_bin = scratch[2];
        need -= scratch[1];
        __syncthreads();
        if (in_bin == 0) { *ok = false; return Pair96{0, 0}; }
        if (j < 8) phi |= (u64)bin << (56 - 8 * j);
        else plo |= bin << (24 - 8 * (j - 8));
        if (in_bin == 1) { ++j; break; }
    }
    if (j < 12) {
        // exactly one string starts with the resolved bytes: fetch the rest of it
        for_each([&](u64 hi, u32 lo) {
            if (pair_matches(hi, lo, phi, plo, j)) { scratch[0] = hi; scratch[1] = lo; }
        });
        __syncthreads();
        phi = scratch[0];
        plo = (u32)scratch[1];
        __syncthreads();
    }
    return Pair96{phi, plo};
}

__device__ __forceinline__ bool pair_le(u64 hi, u32 lo, const Pair96 &p)
{
    return hi < p.hi || (hi == p.hi && lo <= p.lo);
}

// position p of a concatenation of regions -> region index (off[] ascending, off[n] = total)
__device__ __forceinline__ u32 region_of(const u32 *off, u32 n, u32 p)
{
    u32 lo = 0, hi = n;           // answer in [lo, hi): largest b with off[b] <= p
    while (hi - lo > 1) {
        const u32 mid = (lo + hi) >> 1;
        if (off[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------
// finalize: one workgroup turns the short lists into the two cut points and
// the per-unit output offsets.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kFinThreads)
k_finalize(Geom g, PhiloxSeed seed, EncodeCtl *ctl, const u32 *__restrict__ seg_count,
           const u32 *__restrict__ s_idx, const u32 *__restrict__ s_val,
           const u32 *__restrict__ win_sure, const u32 *__restrict__ n_m,
           const u32 *__restrict__ n_b, const u64 *__restrict__ m_key,
           const u32 *__restrict__ m_idx, const u32 *__restrict__ b_mag,
           const u32 *__restrict__ b_idx, u64 *dm_key, u32 *dm_idx, u64 *db_key, u32 *db_idx,
           u32 *__restrict__ unit_base)
{
    __shared__ u32 off_m[kMaxWalkBlocks + 1], off_b[kMaxWalkBlocks + 1];
    __shared__ u32 unit_cnt[kMaxUnits];
    __shared__ u32 h[256];
    __shared__ u64 scan_lds[kFinThreads / kWave + 1];
    __shared__ u64 scratch[4];
    __shared__ u64 st_b_key[kStageB];
    __shared__ u32 st_b_idx[kStageB];
    __shared__ u64 st_m_key[kStageM];
    __shared__ u32 st_m_idx[kStageM];
    __shared__ u32 extra_m, sure_extra;
    __shared__ unsigned long long gt_extra;

    const u32 tid = threadIdx.x;
    const u32 nwaves = kFinThreads / kWave, wave = tid / kWave, lane = lane_id();
    auto unit_of = [&](u32 idx) { return (idx / g.C) / g.SU; };
    // every entry of S, split wavefront by chunk
    auto each_s = [&](auto &&f) {
        for (u32 s = wave; s < g.W; s += nwaves) {
            const u32 n = seg_count[s];
            const u64 at = (u64)s * g.C;
            for (u32 j = lane; j < n; j += kWave) f(s_idx[at + j], s_val[at + j]);
        }
    };

    u64 my_sure = 0, my_super = 0;
    for (u32 u = tid; u < kMaxUnits; u += kFinThreads) {
        const u32 c = u < g.U ? win_sure[u] : 0u;
        unit_cnt[u] = c;
        my_sure += c;
    }
    for (u32 s = tid; s < g.W; s += kFinThreads) my_super += seg_count[s];
    if (tid == 0) { extra_m = 0u; sure_extra = 0u; gt_extra = 0ull; }
    const u32 vm = tid < g.G3 ? n_m[tid] : 0u, vb = tid < g.G3 ? n_b[tid] : 0u;
    const u32 em = (u32)block_exclusive_sum(vm, scan_lds);
    const u32 eb = (u32)block_exclusive_sum(vb, scan_lds);
    off_m[tid] = em;
    off_b[tid] = eb;
    if (tid == kFinThreads - 1) { off_m[kFinThreads] = em + vm; off_b[kFinThreads] = eb + vb; }
    const u64 sure_walk = block_sum(my_sure, scan_lds);
    const u64 superset = block_sum(my_super, scan_lds);
    __syncthreads();
    const u32 n_m0 = off_m[kFinThreads], n_bd = off_b[kFinThreads];

    const u32 bd_hi = ctl->bd_hi, h_shift = ctl->h_shift;
    const u64 c_def = ctl->c_def;
    const u64 need2 = g.r - c_def;
    u32 err = 0, path = 0;
    bool have_t = false, have_k = false, ok = true;
    u32 T = 0, I_star = 0, J_star = 0xFFFFFFFFu, n_mm = 0;
    u64 K_star = ~0ull, count_greater = 0;

    if (ctl->overflow == 0u && need2 >= 1 && need2 <= n_bd) {
        // ---- exact threshold inside the deciding bin --------------------
        const bool b_lds = n_bd <= kStageB;
        u64 *bk = b_lds ? st_b_key : db_key;
        u32 *bi = b_lds ? st_b_idx : db_idx;
        for (u32 p = tid; p < n_bd; p += kFinThreads) {
            const u32 b = region_of(off_b, g.G3, p);
            const u64 at = (u64)b * kListCap + (p - off_b[b]);
            bk[p] = (u64)(bd_hi - b_mag[at]);
            bi[p] = b_idx[at];
        }
        __syncthreads();
        auto each_b = [&](auto &&f) {
            for (u32 p = tid; p < n_bd; p += kFinThreads) f(bk[p], bi[p]);
        };
        const Pair96 tb = block_select96(each_b, need2, (64 - (int)h_shift) / 8, h, scratch, &ok);
        if (ok) {
            have_t = true;
            T = bd_hi - (u32)tb.hi;
            I_star = tb.lo;
            // ---- key lists: walked members + members of the deciding bin
            const bool m_lds = n_m0 + n_bd <= kStageM;
            u64 *mk = m_lds ? st_m_key : dm_key;
            u32 *mi = m_lds ? st_m_idx : dm_idx;
            for (u32 p = tid; p < n_m0; p += kFinThreads) {
                const u32 b = region_of(off_m, g.G3, p);
                const u64 at = (u64)b * kListCap + (p - off_m[b]);
                mk[p] = (m_key[at] - g.K_lo) << g.k_nlz;
                mi[p] = m_idx[at];
            }
            u32 my_gt = 0;
            for (u32 p = tid; p < n_bd; p += kFinThreads) {
                const u64 hi = bk[p];
                const u32 idx = bi[p];
                if (hi < tb.hi) ++my_gt;
                if (!pair_le(hi, idx, tb)) continue;
                bool sure = g.take_all != 0u;
                if (!sure) {
                    const u64 key = sample_key(idx, seed);
                    if (key < g.K_lo) {
                        sure = true;
                    } else if (key <= g.K_hi) {
                        const u32 q = atomicAdd(&extra_m, 1u);
                        mk[n_m0 + q] = (key - g.K_lo) << g.k_nlz;
                        mi[n_m0 + q] = idx;
                    }
                }
                if (sure) { atomicAdd(&unit_cnt[unit_of(idx)], 1u); atomicAdd(&sure_extra, 1u); }
            }
            if (my_gt) atomicAdd(&gt_extra, (unsigned long long)my_gt);
            __syncthreads();
            count_greater = c_def + gt_extra;
            n_mm = n_m0 + extra_m;
            const u64 c_klo = sure_walk + sure_extra;
            if (g.take_all) {
                have_k = true;
            } else if (c_klo < g.k && g.k - c_klo <= n_mm) {
                auto each_m = [&](auto &&f) {
                    for (u32 p = tid; p < n_mm; p += kFinThreads) f(mk[p], mi[p]);
                };
                const Pair96 kb = block_select96(each_m, g.k - c_klo, 0, h, scratch, &ok);
                if (ok) {
                    have_k = true;
                    K_star = (kb.hi >> g.k_nlz) + g.K_lo;
                    J_star = kb.lo;
                    for (u32 p = tid; p < n_mm; p += kFinThreads)
                        if (pair_le(mk[p], mi[p], kb)) atomicAdd(&unit_cnt[unit_of(mi[p])], 1u);
                }
            }
        }
    }

    if (!have_t) {
        // ---- exact threshold by selection over all of S -----------------
        path = 1;
        auto each_mag = [&](auto &&f) {
            each_s([&](u32 idx, u32 bits) { f((u64)(0x7FFFFFFFu - mag_of(bits)), idx); });
        };
        const Pair96 tb = block_select96(each_mag, g.r, 4, h, scratch, &ok);
        if (!ok) err |= kErrSelect;
        T = 0x7FFFFFFFu - (u32)tb.hi;
        I_star = tb.lo;
        u64 my_gt = 0;
        each_s([&](u32, u32 bits) { if (mag_of(bits) > T) ++my_gt; });
        count_greater = block_sum(my_gt, scan_lds);
    }
    auto is_member = [&](u32 idx, u32 bits) {
        const u32 m = mag_of(bits);
        return m > T || (m == T && idx <= I_star);
    };
    if (!have_k) {
        // ---- exact key cut and per-unit winners by selection over S -----
        path = 1;
        __syncthreads();
        for (u32 u = tid; u < kMaxUnits; u += kFinThreads) unit_cnt[u] = 0u;
        if (!g.take_all) {
            auto each_key = [&](auto &&f) {
                each_s([&](u32 idx, u32 bits) {
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
        each_s([&](u32 idx, u32 bits) {
            if (is_member(idx, bits) &&
                (g.take_all || pair_le(sample_key(idx, seed), idx, kcut)))
                atomicAdd(&unit_cnt[unit_of(idx)], 1u);
        });
    }
    __syncthreads();

    // ---- output offset of every unit ------------------------------------
    constexpr u32 per = kMaxUnits / kFinThreads;
    u32 c[per];
    u64 mine = 0;
#pragma unroll
    for (u32 q = 0; q < per; ++q) { c[q] = unit_cnt[tid * per + q]; mine += c[q]; }
    u64 run = block_exclusive_sum(mine, scan_lds);
    const u64 total = scan_lds[kFinThreads / kWave];
#pragma unroll
    for (u32 q = 0; q < per; ++q) {
        const u32 u = tid * per + q;
        if (u < g.U) unit_base[u] = (u32)run;
        run += c[q];
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
        ctl->superset = superset;
        ctl->count_greater = count_greater;
        ctl->ties = g.r - count_greater;
    }
}

// ---------------------------------------------------------------------------
// emit: members of the top-r set whose (key, index) is at or below the cut
// -> the message in index order; residual at the sent positions <- a - a.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kWalkThreads)
k_emit(Geom g, PhiloxSeed seed, const EncodeCtl *__restrict__ ctl,
       const u32 *__restrict__ seg_count, const u32 *__restrict__ s_idx,
       const u32 *__restrict__ s_val, const u32 *__restrict__ unit_base,
       u32 *__restrict__ out_idx, float *__restrict__ out_val, float *__restrict__ residual)
{
    const u32 u = blockIdx.x * kWalkWaves + threadIdx.x / kWave;
    if (u >= g.U) return;
    const u32 lane = lane_id();
    const u32 T = ctl->T, I_star = ctl->I_star;
    const Pair96 kcut{ctl->K_star, ctl->J_star};
    const u64 below = lanes_below();
    u64 run = unit_base[u];
    const u32 s_end = (u + 1) * g.SU < g.W ? (u + 1) * g.SU : g.W;
    for (u32 s = u * g.SU; s < s_end; ++s) {
        const u32 n = seg_count[s];
        const u64 at = (u64)s * g.C;
        for (u32 j0 = 0; j0 < n; j0 += kWave) {
            const u32 j = j0 + lane;
            bool win = false;
            u32 idx = 0, bits = 0;
            if (j < n) {
                idx = s_idx[at + j];
                bits = s_val[at + j];
                const u32 m = mag_of(bits);
                win = m > T || (m == T && idx <= I_star);
                if (win && !g.take_all) win = pair_le(sample_key(idx, seed), idx, kcut);
            }
            const u64 mask = __ballot(win);
            if (win) {
                const u64 pos = run + popc64(mask & below);
                if (pos < g.k) {
                    const float v = __uint_as_float(bits);
                    out_idx[pos] = idx;
                    out_val[pos] = v;
                    residual[idx] = v - v;
                }
            }
            run += popc64(mask);
        }
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
}  // namespace

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

extern "C" int rtopk_encode(const float *grad, float *residual, uint64_t d, uint64_t r,
                            uint64_t k, uint64_t seed, uint64_t step, uint32_t *out_idx,
                            float *out_val, void *workspace, uint64_t workspace_bytes,
                            void *stream_v)
{
    if (!grad || !residual || !out_idx || !out_val) return RTOPK_EINVAL;
    const int rc = check_sizes(d, r, k);
    if (rc) return rc;
    {
        const uintptr_t g0 = (uintptr_t)grad, m0 = (uintptr_t)residual;
        if (g0 < m0 + d * 4 && m0 < g0 + d * 4) return RTOPK_EINVAL;
    }
    const Geom g = make_geom(d, r, k);
    const EncodeLayout L = make_layout(g);
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < L.total)
        return RTOPK_EWORKSPACE;

    hipStream_t stream = (hipStream_t)stream_v;
    char *ws = (char *)workspace;
    EncodeCtl *ctl = (EncodeCtl *)(ws + L.ctl);
    u32 *hist1 = (u32 *)(ws + L.hist1), *hist2 = (u32 *)(ws + L.hist2);
    u32 *seg_count = (u32 *)(ws + L.seg_count), *win_sure = (u32 *)(ws + L.win_sure);
    u32 *unit_base = (u32 *)(ws + L.unit_base);
    u32 *n_m = (u32 *)(ws + L.n_m), *n_b = (u32 *)(ws + L.n_b);
    u64 *m_key = (u64 *)(ws + L.m_key), *dm_key = (u64 *)(ws + L.dm_key);
    u64 *db_key = (u64 *)(ws + L.db_key);
    u32 *m_idx = (u32 *)(ws + L.m_idx), *b_mag = (u32 *)(ws + L.b_mag);
    u32 *b_idx = (u32 *)(ws + L.b_idx), *dm_idx = (u32 *)(ws + L.dm_idx);
    u32 *db_idx = (u32 *)(ws + L.db_idx);
    u32 *s_idx = (u32 *)(ws + L.s_idx), *s_val = (u32 *)(ws + L.s_val);

    const PhiloxSeed ps{(u32)seed, (u32)(seed >> 32), (u32)step, (u32)(step >> 32)};
    const bool vec4 = (((uintptr_t)grad | (uintptr_t)residual) & 15u) == 0;
    const bool rvec4 = ((uintptr_t)residual & 15u) == 0;

    const TraceRequest trace = g_trace;
    g_trace = TraceRequest{};
    StageScope whole(trace, RTOPK_STAGE_ALL, stream);

    {
        StageScope sc(trace, RTOPK_STAGE_INIT, stream);
        const u32 words = (u32)(L.zero_bytes / 4);
        k_init<<<(words + 255) / 256, 256, 0, stream>>>((u32 *)ws, words);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_FUSED, stream);
        const u64 per_block = (u64)kFusedThreads * (vec4 ? 16 : 4);
        u64 want = (d + per_block - 1) / per_block;
        const unsigned grid = (unsigned)(want < 1 ? 1 : (want > 512 ? 512 : want));
        if (vec4)
            k_fused_add_hist<true><<<grid, kFusedThreads, 0, stream>>>(grad, residual, d, hist1);
        else
            k_fused_add_hist<false><<<grid, kFusedThreads, 0, stream>>>(grad, residual, d, hist1);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_SCAN, stream);
        const unsigned grid = (g.W + kWalkWaves - 1) / kWalkWaves;
        if (rvec4)
            k_scan<true><<<grid, kWalkThreads, 0, stream>>>(residual, g, ctl, hist1, hist2,
                                                            seg_count, s_idx, s_val);
        else
            k_scan<false><<<grid, kWalkThreads, 0, stream>>>(residual, g, ctl, hist1, hist2,
                                                             seg_count, s_idx, s_val);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_CLASSIFY, stream);
        k_classify<<<g.G3, kWalkThreads, 0, stream>>>(g, ps, ctl, hist2, seg_count, s_idx, s_val,
                                                      win_sure, n_m, n_b, m_key, m_idx, b_mag,
                                                      b_idx);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_FINALIZE, stream);
        k_finalize<<<1, kFinThreads, 0, stream>>>(g, ps, ctl, seg_count, s_idx, s_val, win_sure,
                                                  n_m, n_b, m_key, m_idx, b_mag, b_idx, dm_key,
                                                  dm_idx, db_key, db_idx, unit_base);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_EMIT, stream);
        k_emit<<<g.G3, kWalkThreads, 0, stream>>>(g, ps, ctl, seg_count, s_idx, s_val, unit_base,
                                                  out_idx, out_val, residual);
        RTOPK_LAUNCH_CHECK();
    }
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
    host_out->error_flags = c.err;
    host_out->path = c.path;
    host_out->threshold_bits = c.T;
    host_out->boundary_list_size = c.n_b;
    host_out->count_greater = c.count_greater;
    host_out->ties_taken = c.ties;
    host_out->superset_size = c.superset;
    host_out->key_list_size = c.n_m;
    return RTOPK_OK;
}
