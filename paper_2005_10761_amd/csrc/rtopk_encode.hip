// rtopk_encode: one node-side step of Algorithm 1 (error compensation, the
// rTop-k operator of Definition 3, residual write-back) as a chain of gfx950
// kernels. All cross-kernel state lives in the caller's workspace.
//
// Pipeline (d = vector length, S = a compacted superset of the top-r set):
//   init            zero the control block, histograms and scan status words
//   fused_add_hist  a = g + m, stored into the residual buffer; histogram of
//                   the top 12 magnitude bits; the last workgroup out picks
//                   the bucket that holds the r-th largest magnitude
//   compact_superset  all entries in that bucket or above -> S, index order
//   hist_pass<2>, hist_pass<3>  next 11 and last 8 magnitude bits, restricted
//                   to the running prefix; last workgroup out picks
//   select_top_r    entries above the threshold plus the lowest-index ties
//                   -> the r candidates, index order
//   key_hist        Philox keys of the candidates, histogram of the top 12
//                   key bits; last workgroup out picks the deciding bucket
//   key_collect     candidates in the deciding bucket -> small list; the last
//                   workgroup out finds the exact k-th smallest (key, index)
//   emit            candidates at or below it -> message, index order;
//                   residual at sent positions <- a - a
// Every compaction is order preserving (chained scan with look-back), so the
// message comes out sorted by index without any sort.
#include "rtopk_common.h"
#include "../../include/rtopk.h"

namespace rtopk {

// ---------------------------------------------------------------------------
// digits of the 31-bit magnitude pattern, most significant first
// ---------------------------------------------------------------------------
constexpr int kBits1 = 12, kBits2 = 11, kBits3 = 8;
constexpr int kShift1 = 19, kShift2 = 8;
constexpr int kBins1 = 1 << kBits1, kBins2 = 1 << kBits2, kBins3 = 1 << kBits3;
constexpr int kKeyBits = 12, kKeyBins = 1 << kKeyBits, kKeyShift = 64 - kKeyBits;

constexpr int kTileThreads = 256;             // ordered-compaction kernels
constexpr int kTileElems = 4096;              // 16 elements per thread
constexpr int kTileWaves = kTileThreads / kWave;

constexpr u32 kModeSuperset = 0, kModeFull = 1;

struct EncodeCtl {
    u32 err;
    u32 mode;
    u32 ticket_compact, ticket_select, ticket_emit;
    u32 done_fused, done_hist2, done_hist3, done_keyhist, done_collect;
    u32 prefix;        // resolved high bits of the threshold pattern
    u32 threshold;     // full 31-bit pattern once pass 3 has picked
    u64 need;          // how many entries are still to be taken inside the prefix bucket
    u64 count_greater; // entries known to be strictly above the prefix bucket
    u64 superset;      // size of S
    u64 ties;          // entries equal to the threshold that belong to the top-r set
    u32 key_digit;     // deciding top digit of the sampling keys
    u32 key_list;      // entries collected from that bucket
    u64 key_need;      // rank (1-based) of the deciding key inside the bucket
    u64 key_star;      // the k-th smallest (key, index): key ...
    u32 idx_star;      // ... and index
    u32 pad;
};

struct EncodeLayout {
    u64 ctl, hist1, hist2, hist3, histk;
    u64 st_compact, st_sel_gt, st_sel_eq, st_emit;
    u64 zero_bytes;                       // [0, zero_bytes) is cleared by init
    u64 s_idx, s_val, cand_idx, cand_val, m_key, m_idx;
    u64 total;
    u64 cap_s;
    u32 tiles_full, tiles_cand;
};

static EncodeLayout make_layout(u64 d, u64 r)
{
    EncodeLayout L{};
    u64 cap = 2 * r + 4096;
    if (cap < d / 8) cap = d / 8;
    if (cap > d) cap = d;
    L.cap_s = cap;
    L.tiles_full = (u32)((d + kTileElems - 1) / kTileElems);
    L.tiles_cand = (u32)((r + kTileElems - 1) / kTileElems);
    u64 o = 0;
    auto take = [&](u64 bytes) { u64 at = o; o = align_up(o + bytes, 256); return at; };
    L.ctl = take(sizeof(EncodeCtl));
    L.hist1 = take(kBins1 * 4);
    L.hist2 = take(kBins2 * 4);
    L.hist3 = take(kBins3 * 4);
    L.histk = take(kKeyBins * 4);
    L.st_compact = take((u64)L.tiles_full * 8);
    L.st_sel_gt = take((u64)L.tiles_full * 8);
    L.st_sel_eq = take((u64)L.tiles_full * 8);
    L.st_emit = take((u64)L.tiles_cand * 8);
    L.zero_bytes = o;
    L.s_idx = take(cap * 4);
    L.s_val = take(cap * 4);
    L.cand_idx = take(r * 4);
    L.cand_val = take(r * 4);
    L.m_key = take(r * 8);
    L.m_idx = take(r * 4);
    L.total = o;
    return L;
}

__device__ __forceinline__ u32 mag_of(u32 bits) { return bits & 0x7FFFFFFFu; }

// ---------------------------------------------------------------------------
// block-wide exclusive prefix sum of one u64 per thread (thread order)
// ---------------------------------------------------------------------------
__device__ __forceinline__ u64 block_exclusive_sum(u64 v, u64 *lds /* >= 17 words */)
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
    }
    __syncthreads();
    const u64 res = lds[wave] + inc - v;
    __syncthreads();
    return res;
}

// Whole workgroup: find the bucket b with  #(bins above b) < need <= #(bins >= b)
// when walking the bins from the top (descending = true) or from the bottom.
// Returns b and the population strictly before it in walking order.
template <bool kDescending>
__device__ __forceinline__ void block_pick(const u32 *hist, int nbins, u64 need,
                                           u32 *out_bin, u64 *out_before, u64 *lds)
{
    const int per = (nbins + (int)blockDim.x - 1) / (int)blockDim.x;
    const int first = (int)threadIdx.x * per;      // position in walking order
    u64 mine = 0;
    for (int q = 0; q < per; ++q) {
        const int pos = first + q;
        if (pos < nbins) mine += hist[kDescending ? nbins - 1 - pos : pos];
    }
    const u64 before = block_exclusive_sum(mine, lds);
    if (before < need && need <= before + mine) {
        u64 run = before;
        for (int q = 0; q < per; ++q) {
            const int pos = first + q;
            if (pos >= nbins) break;
            const int bin = kDescending ? nbins - 1 - pos : pos;
            const u64 h = hist[bin];
            if (run + h >= need) { *out_bin = (u32)bin; *out_before = run; break; }
            run += h;
        }
    }
}

// ---------------------------------------------------------------------------
// init: clear everything the later kernels expect to start at zero
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_init(u32 *zero_base, u64 words)
{
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < words;
         i += (u64)gridDim.x * blockDim.x)
        zero_base[i] = 0u;
}

// ---------------------------------------------------------------------------
// fused residual add + first histogram (12d bytes of HBM traffic)
// ---------------------------------------------------------------------------
constexpr int kFusedThreads = 1024;
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool kVec4>
__global__ void __launch_bounds__(kFusedThreads)
k_fused_add_hist(const float *__restrict__ grad, float *__restrict__ residual, u64 d, u64 r,
                 u64 cap_s, EncodeCtl *ctl, u32 *hist1)
{
    __shared__ u32 h[kBins1];
    __shared__ u64 scan_lds[kFusedThreads / kWave + 1];
    __shared__ u32 flag;
    for (int b = threadIdx.x; b < kBins1; b += kFusedThreads) h[b] = 0u;
    __syncthreads();

    auto count = [&](u32 bits) { atomicAdd(&h[mag_of(bits) >> kShift1], 1u); };

    if (kVec4) {
        const u64 nvec = d / 4;
        const f32x4 *g4 = reinterpret_cast<const f32x4 *>(grad);
        f32x4 *m4 = reinterpret_cast<f32x4 *>(residual);
        const u64 stride = (u64)gridDim.x * kFusedThreads;
        u64 v = (u64)blockIdx.x * kFusedThreads + threadIdx.x;
        auto body = [&](const f32x4 &g, const f32x4 &m, u64 at) {
            const f32x4 a = g + m;
            m4[at] = a;
            const u32 b0 = __float_as_uint(a.x), b1 = __float_as_uint(a.y),
                      b2 = __float_as_uint(a.z), b3 = __float_as_uint(a.w);
            const u32 d0 = mag_of(b0) >> kShift1, d1 = mag_of(b1) >> kShift1,
                      d2 = mag_of(b2) >> kShift1, d3 = mag_of(b3) >> kShift1;
            // runs of equal digits (zero rows, constant blocks): one add per wave
            const u32 lead = __builtin_amdgcn_readfirstlane(d0);
            const bool same = (d0 == lead) & (d1 == lead) & (d2 == lead) & (d3 == lead);
            const u64 same_mask = __ballot(same);
            const u64 active = __ballot(true);
            if (same_mask == active) {
                if (lane_id() == (u32)(__ffsll((unsigned long long)active) - 1))
                    atomicAdd(&h[lead], 4u * (u32)__popcll(active));
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
            count(__float_as_uint(a));
        }
    } else {
        const u64 stride = (u64)gridDim.x * kFusedThreads;
        for (u64 i = (u64)blockIdx.x * kFusedThreads + threadIdx.x; i < d; i += stride) {
            const float a = grad[i] + residual[i];
            residual[i] = a;
            count(__float_as_uint(a));
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins1; b += kFusedThreads) {
        const u32 c = h[b];
        if (c) atomicAdd(&hist1[b], c);
    }

    if (last_block_done(&ctl->done_fused, &flag)) {
        __shared__ u32 bin;
        __shared__ u64 before;
        block_pick<true>(hist1, kBins1, r, &bin, &before, scan_lds);
        __syncthreads();
        if (threadIdx.x == 0) {
            const u64 s = before + hist1[bin];
            ctl->prefix = bin << kShift1;
            ctl->count_greater = before;
            ctl->need = r - before;
            ctl->superset = s;
            ctl->mode = (s <= cap_s) ? kModeSuperset : kModeFull;
        }
    }
}

// ---------------------------------------------------------------------------
// ordered offsets inside one 4096-element tile (256 threads, ROWS rows)
// element order: row, then thread, then position inside the thread's vector.
// cnt[j] may pack two 16-bit counters; totals stay below 2^16 each.
// lds: ROWS * kTileWaves + 1 words.
// ---------------------------------------------------------------------------
template <int ROWS>
__device__ __forceinline__ void tile_offsets(const u32 (&cnt)[ROWS], u32 (&off)[ROWS],
                                             u32 &tile_total, u32 *lds)
{
    constexpr int nseg = ROWS * kTileWaves;
    static_assert(nseg <= kWave, "segment scan is done by one wave");
    const u32 lane = lane_id(), wave = threadIdx.x / kWave;
    u32 lane_excl[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        u32 total = 0;
        lane_excl[j] = 0;
        if (__ballot(cnt[j] != 0u) != 0ull) {
            const u32 inc = wave_inclusive_sum(cnt[j]);
            lane_excl[j] = inc - cnt[j];
            total = __shfl(inc, kWave - 1, kWave);
        }
        if (lane == 0) lds[j * kTileWaves + wave] = total;
    }
    __syncthreads();
    if (wave == 0) {
        const u32 v = lane < (u32)nseg ? lds[lane] : 0u;
        const u32 inc = wave_inclusive_sum(v);
        if (lane < (u32)nseg) lds[lane] = inc - v;
        if (lane == (u32)nseg - 1) lds[nseg] = inc;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < ROWS; ++j) off[j] = lds[j * kTileWaves + wave] + lane_excl[j];
    tile_total = lds[nseg];
}

__device__ __forceinline__ u32 claim_tile(u32 *ticket, u32 *lds_slot)
{
    __syncthreads();
    if (threadIdx.x == 0) *lds_slot = atomicAdd(ticket, 1u);
    __syncthreads();
    return *lds_slot;
}

// ---------------------------------------------------------------------------
// compact_superset: every entry whose top digit is at or above the picked
// bucket -> (S_idx, S_val) in index order. Reads a once (4d bytes).
// ---------------------------------------------------------------------------
template <bool kVec4>
__global__ void __launch_bounds__(kTileThreads)
k_compact_superset(const float *__restrict__ a, u64 d, EncodeCtl *ctl, u64 *status,
                   u32 *__restrict__ s_idx, u32 *__restrict__ s_val, u64 cap_s)
{
    constexpr int VEC = kVec4 ? 4 : 1;
    constexpr int ROWS = kTileElems / (kTileThreads * VEC);
    __shared__ u32 lds[ROWS * kTileWaves + 1];
    __shared__ u32 slot;
    __shared__ u64 base_lds;
    if (ctl->mode != kModeSuperset) return;
    const u32 digit_min = ctl->prefix >> kShift1;
    const u32 tile = claim_tile(&ctl->ticket_compact, &slot);
    const u64 tile_base = (u64)tile * kTileElems;

    u32 bits[ROWS][VEC];
    u32 cnt[ROWS], off[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const u64 e0 = tile_base + (u64)j * (kTileThreads * VEC) + (u64)threadIdx.x * VEC;
        cnt[j] = 0;
        bool loaded = false;
        if constexpr (kVec4) {
            if (e0 + 3 < d) {
                const float4 v = *reinterpret_cast<const float4 *>(a + e0);
                bits[j][0] = __float_as_uint(v.x);
                bits[j][1] = __float_as_uint(v.y);
                bits[j][2] = __float_as_uint(v.z);
                bits[j][3] = __float_as_uint(v.w);
                loaded = true;
            }
        }
        if (!loaded) {
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                bits[j][e] = (e0 + e < d) ? __float_as_uint(a[e0 + e]) : 0u;
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const u64 i = e0 + e;
            const bool hit = (i < d) && ((mag_of(bits[j][e]) >> kShift1) >= digit_min);
            cnt[j] += hit ? 1u : 0u;
        }
    }
    u32 tile_total;
    tile_offsets<ROWS>(cnt, off, tile_total, lds);
    if (threadIdx.x < kWave) {
        const u64 base = lookback_exclusive(status, tile, tile_total, &ctl->err);
        if (threadIdx.x == 0) base_lds = base;
    }
    __syncthreads();
    const u64 base = base_lds;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        if (cnt[j] == 0) continue;
        const u64 e0 = tile_base + (u64)j * (kTileThreads * VEC) + (u64)threadIdx.x * VEC;
        u64 pos = base + off[j];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const u64 i = e0 + e;
            if ((i < d) && ((mag_of(bits[j][e]) >> kShift1) >= digit_min)) {
                if (pos < cap_s) { s_idx[pos] = (u32)i; s_val[pos] = bits[j][e]; }
                ++pos;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// hist_pass<P>: histogram of digit P over the entries whose higher digits
// equal the running prefix; source is S (superset mode) or a itself.
// ---------------------------------------------------------------------------
constexpr int kHistThreads = 256;

template <int PASS>
__global__ void __launch_bounds__(kHistThreads)
k_hist_pass(const float *__restrict__ a, u64 d, const u32 *__restrict__ s_val,
            EncodeCtl *ctl, u32 *hist)
{
    constexpr int nbins = PASS == 2 ? kBins2 : kBins3;
    constexpr int hi_shift = PASS == 2 ? kShift1 : kShift2;   // bits above this digit
    constexpr int lo_shift = PASS == 2 ? kShift2 : 0;
    __shared__ u32 h[nbins];
    __shared__ u64 scan_lds[kHistThreads / kWave + 1];
    __shared__ u32 flag;
    for (int b = threadIdx.x; b < nbins; b += kHistThreads) h[b] = 0u;
    __syncthreads();
    const bool superset = ctl->mode == kModeSuperset;
    const u64 n = superset ? ctl->superset : d;
    const u32 *src = superset ? s_val : reinterpret_cast<const u32 *>(a);
    const u32 want = ctl->prefix >> hi_shift;
    bool any = false;
    for (u64 i = (u64)blockIdx.x * kHistThreads + threadIdx.x; i < n;
         i += (u64)gridDim.x * kHistThreads) {
        const u32 m = mag_of(src[i]);
        if ((m >> hi_shift) == want) {
            atomicAdd(&h[(m >> lo_shift) & (nbins - 1)], 1u);
            any = true;
        }
    }
    if (__syncthreads_or(any ? 1 : 0)) {
        for (int b = threadIdx.x; b < nbins; b += kHistThreads) {
            const u32 c = h[b];
            if (c) atomicAdd(&hist[b], c);
        }
    }
    u32 *done = PASS == 2 ? &ctl->done_hist2 : &ctl->done_hist3;
    if (last_block_done(done, &flag)) {
        __shared__ u32 bin;
        __shared__ u64 before;
        block_pick<true>(hist, nbins, ctl->need, &bin, &before, scan_lds);
        __syncthreads();
        if (threadIdx.x == 0) {
            const u32 prefix = ctl->prefix | (bin << lo_shift);
            ctl->prefix = prefix;
            ctl->count_greater += before;
            ctl->need -= before;
            if (PASS == 3) {
                ctl->threshold = prefix;
                ctl->ties = ctl->need;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// select_top_r: entries above the threshold, plus the `ties` lowest-index
// entries equal to it -> r candidates in index order.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kTileThreads)
k_select_top_r(const float *__restrict__ a, u64 d, const u32 *__restrict__ s_idx,
               const u32 *__restrict__ s_val, EncodeCtl *ctl, u64 *st_gt, u64 *st_eq,
               u32 *__restrict__ cand_idx, u32 *__restrict__ cand_val, u64 r)
{
    constexpr int ROWS = kTileElems / kTileThreads;   // 16 scalar rows
    __shared__ u32 lds[ROWS * kTileWaves + 1];
    __shared__ u32 slot;
    __shared__ u64 base_lds[2];
    const bool superset = ctl->mode == kModeSuperset;
    const u64 n = superset ? ctl->superset : d;
    const u32 *src = superset ? s_val : reinterpret_cast<const u32 *>(a);
    const u32 thr = ctl->threshold;
    const u64 ties = ctl->ties;
    const u64 ntiles = (n + kTileElems - 1) / kTileElems;

    while (true) {
        const u32 tile = claim_tile(&ctl->ticket_select, &slot);
        if (tile >= ntiles) break;
        const u64 tile_base = (u64)tile * kTileElems;
        u32 bits[ROWS], cnt[ROWS], off[ROWS];
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const u64 i = tile_base + (u64)j * kTileThreads + threadIdx.x;
            bits[j] = 0u;
            cnt[j] = 0u;
            if (i < n) {
                bits[j] = src[i];
                const u32 m = mag_of(bits[j]);
                cnt[j] = (m > thr ? 1u : 0u) | (m == thr ? 0x10000u : 0u);
            }
        }
        u32 tile_total;
        tile_offsets<ROWS>(cnt, off, tile_total, lds);
        if (threadIdx.x < kWave) {
            const u64 bg = lookback_exclusive(st_gt, tile, tile_total & 0xFFFFu, &ctl->err);
            const u64 be = lookback_exclusive(st_eq, tile, tile_total >> 16, &ctl->err);
            if (threadIdx.x == 0) { base_lds[0] = bg; base_lds[1] = be; }
        }
        __syncthreads();
        const u64 base_gt = base_lds[0], base_eq = base_lds[1];
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            if (cnt[j] == 0u) continue;
            const u64 gt_before = base_gt + (off[j] & 0xFFFFu);
            const u64 eq_before = base_eq + (off[j] >> 16);
            const bool take = (cnt[j] & 1u) || eq_before < ties;
            if (take) {
                const u64 pos = gt_before + (eq_before < ties ? eq_before : ties);
                if (pos < r) {
                    const u64 i = tile_base + (u64)j * kTileThreads + threadIdx.x;
                    cand_idx[pos] = superset ? s_idx[i] : (u32)i;
                    cand_val[pos] = bits[j];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// key_hist: histogram of the top key digit over the r candidates; the last
// workgroup out picks the bucket holding the k-th smallest key.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kHistThreads)
k_key_hist(const u32 *__restrict__ cand_idx, u64 r, u64 k, PhiloxSeed seed,
           EncodeCtl *ctl, u32 *histk)
{
    __shared__ u32 h[kKeyBins];
    __shared__ u64 scan_lds[kHistThreads / kWave + 1];
    __shared__ u32 flag;
    for (int b = threadIdx.x; b < kKeyBins; b += kHistThreads) h[b] = 0u;
    __syncthreads();
    for (u64 i = (u64)blockIdx.x * kHistThreads + threadIdx.x; i < r;
         i += (u64)gridDim.x * kHistThreads) {
        const u64 key = sample_key(cand_idx[i], seed);
        atomicAdd(&h[(u32)(key >> kKeyShift)], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kKeyBins; b += kHistThreads) {
        const u32 c = h[b];
        if (c) atomicAdd(&histk[b], c);
    }
    if (last_block_done(&ctl->done_keyhist, &flag)) {
        __shared__ u32 bin;
        __shared__ u64 before;
        block_pick<false>(histk, kKeyBins, k, &bin, &before, scan_lds);
        __syncthreads();
        if (threadIdx.x == 0) {
            ctl->key_digit = bin;
            ctl->key_need = k - before;
        }
    }
}

// ---------------------------------------------------------------------------
// key_collect: candidates whose key falls in the deciding bucket -> list M
// (unordered); the last workgroup out finds the key_need-th smallest
// (key, index) of M by a byte-wise radix select over the 96-bit pair.
// ---------------------------------------------------------------------------
__device__ __forceinline__ u32 pair_byte(u64 key, u32 idx, int j /* 0 = most significant */)
{
    // bytes of the 96-bit string key:idx
    return j < 8 ? (u32)(key >> (56 - 8 * j)) & 0xFFu : (idx >> (24 - 8 * (j - 8))) & 0xFFu;
}

__device__ __forceinline__ bool pair_matches(u64 key, u32 idx, u64 pkey, u32 pidx, int nbytes)
{
    // do the first nbytes bytes of key:idx equal those of pkey:pidx ?
    if (nbytes <= 0) return true;
    if (nbytes >= 8) {
        if (key != pkey) return false;
        const int rest = nbytes - 8;
        return rest == 0 || (idx >> (32 - 8 * rest)) == (pidx >> (32 - 8 * rest));
    }
    return (key >> (64 - 8 * nbytes)) == (pkey >> (64 - 8 * nbytes));
}

__global__ void __launch_bounds__(kHistThreads)
k_key_collect(const u32 *__restrict__ cand_idx, u64 r, PhiloxSeed seed, EncodeCtl *ctl,
              u64 *__restrict__ m_key, u32 *__restrict__ m_idx)
{
    __shared__ u32 h[256];
    __shared__ u64 scan_lds[kHistThreads / kWave + 1];
    __shared__ u32 flag;
    const u32 want = ctl->key_digit;
    for (u64 i = (u64)blockIdx.x * kHistThreads + threadIdx.x; i < r;
         i += (u64)gridDim.x * kHistThreads) {
        const u32 idx = cand_idx[i];
        const u64 key = sample_key(idx, seed);
        if ((u32)(key >> kKeyShift) == want) {
            const u32 at = atomicAdd(&ctl->key_list, 1u);
            m_key[at] = key;
            m_idx[at] = idx;
        }
    }
    if (!last_block_done(&ctl->done_collect, &flag)) return;

    const u32 n = load_agent(&ctl->key_list);
    u64 need = ctl->key_need;
    u64 pkey = 0;
    u32 pidx = 0;
    __shared__ u32 bin;
    __shared__ u64 before;
    // byte 0 and the high half of byte 1 are shared by the whole bucket, so
    // start at byte 1 with byte 0 already known
    pkey = (u64)want << kKeyShift;
    for (int j = 1; j < 12; ++j) {
        for (int b = threadIdx.x; b < 256; b += kHistThreads) h[b] = 0u;
        __syncthreads();
        for (u32 e = threadIdx.x; e < n; e += kHistThreads) {
            const u64 key = m_key[e];
            const u32 idx = m_idx[e];
            if (pair_matches(key, idx, pkey, pidx, j)) atomicAdd(&h[pair_byte(key, idx, j)], 1u);
        }
        __syncthreads();
        block_pick<false>(h, 256, need, &bin, &before, scan_lds);
        __syncthreads();
        need -= before;
        if (j < 8) pkey |= (u64)bin << (56 - 8 * j);
        else pidx |= bin << (24 - 8 * (j - 8));
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        ctl->key_star = pkey;
        ctl->idx_star = pidx;
    }
}

// ---------------------------------------------------------------------------
// emit: candidates with (key, index) <= (key*, index*) -> the message, in
// index order; residual at the sent positions <- a - a.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kTileThreads)
k_emit(const u32 *__restrict__ cand_idx, const u32 *__restrict__ cand_val, u64 r, u64 k,
       PhiloxSeed seed, EncodeCtl *ctl, u64 *status, u32 *__restrict__ out_idx,
       float *__restrict__ out_val, float *__restrict__ residual)
{
    constexpr int ROWS = kTileElems / kTileThreads;
    __shared__ u32 lds[ROWS * kTileWaves + 1];
    __shared__ u32 slot;
    __shared__ u64 base_lds;
    const u64 kstar = ctl->key_star;
    const u32 istar = ctl->idx_star;
    const u32 tile = claim_tile(&ctl->ticket_emit, &slot);
    const u64 tile_base = (u64)tile * kTileElems;
    u32 idx[ROWS], cnt[ROWS], off[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const u64 i = tile_base + (u64)j * kTileThreads + threadIdx.x;
        cnt[j] = 0u;
        idx[j] = 0u;
        if (i < r) {
            idx[j] = cand_idx[i];
            const u64 key = sample_key(idx[j], seed);
            cnt[j] = (key < kstar || (key == kstar && idx[j] <= istar)) ? 1u : 0u;
        }
    }
    u32 tile_total;
    tile_offsets<ROWS>(cnt, off, tile_total, lds);
    if (threadIdx.x < kWave) {
        const u64 base = lookback_exclusive(status, tile, tile_total, &ctl->err);
        if (threadIdx.x == 0) base_lds = base;
    }
    __syncthreads();
    const u64 base = base_lds;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        if (cnt[j] == 0u) continue;
        const u64 pos = base + off[j];
        if (pos < k) {
            const u64 i = tile_base + (u64)j * kTileThreads + threadIdx.x;
            const float v = __uint_as_float(cand_val[i]);
            out_idx[pos] = idx[j];
            out_val[pos] = v;
            residual[idx[j]] = v - v;
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
    *bytes = make_layout(d, r).total;
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
    const EncodeLayout L = make_layout(d, r);
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < L.total)
        return RTOPK_EWORKSPACE;

    hipStream_t stream = (hipStream_t)stream_v;
    char *ws = (char *)workspace;
    EncodeCtl *ctl = (EncodeCtl *)(ws + L.ctl);
    u32 *hist1 = (u32 *)(ws + L.hist1), *hist2 = (u32 *)(ws + L.hist2);
    u32 *hist3 = (u32 *)(ws + L.hist3), *histk = (u32 *)(ws + L.histk);
    u64 *st_compact = (u64 *)(ws + L.st_compact), *st_gt = (u64 *)(ws + L.st_sel_gt);
    u64 *st_eq = (u64 *)(ws + L.st_sel_eq), *st_emit = (u64 *)(ws + L.st_emit);
    u32 *s_idx = (u32 *)(ws + L.s_idx), *s_val = (u32 *)(ws + L.s_val);
    u32 *cand_idx = (u32 *)(ws + L.cand_idx), *cand_val = (u32 *)(ws + L.cand_val);
    u64 *m_key = (u64 *)(ws + L.m_key);
    u32 *m_idx = (u32 *)(ws + L.m_idx);

    const PhiloxSeed ps{(u32)seed, (u32)(seed >> 32), (u32)step, (u32)(step >> 32)};
    const bool vec4 = (((uintptr_t)grad | (uintptr_t)residual) & 15u) == 0;

    auto clamp_grid = [](u64 want, u64 lo, u64 hi) {
        return (unsigned)(want < lo ? lo : (want > hi ? hi : want));
    };
    const TraceRequest trace = g_trace;
    g_trace = TraceRequest{};
    StageScope whole(trace, RTOPK_STAGE_ALL, stream);

    {
        StageScope sc(trace, RTOPK_STAGE_INIT, stream);
        const u64 words = L.zero_bytes / 4;
        k_init<<<clamp_grid((words + 255) / 256, 1, 1024), 256, 0, stream>>>((u32 *)ws, words);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_FUSED, stream);
        const u64 per_block = (u64)kFusedThreads * (vec4 ? 16 : 4);
        const unsigned grid = clamp_grid((d + per_block - 1) / per_block, 1, 512);
        if (vec4)
            k_fused_add_hist<true><<<grid, kFusedThreads, 0, stream>>>(grad, residual, d, r,
                                                                      L.cap_s, ctl, hist1);
        else
            k_fused_add_hist<false><<<grid, kFusedThreads, 0, stream>>>(grad, residual, d, r,
                                                                       L.cap_s, ctl, hist1);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_COMPACT, stream);
        const bool rvec4 = ((uintptr_t)residual & 15u) == 0;
        if (rvec4)
            k_compact_superset<true><<<L.tiles_full, kTileThreads, 0, stream>>>(
                residual, d, ctl, st_compact, s_idx, s_val, L.cap_s);
        else
            k_compact_superset<false><<<L.tiles_full, kTileThreads, 0, stream>>>(
                residual, d, ctl, st_compact, s_idx, s_val, L.cap_s);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_REFINE, stream);
        const unsigned grid = clamp_grid((L.cap_s + 2047) / 2048, 1, 512);
        k_hist_pass<2><<<grid, kHistThreads, 0, stream>>>(residual, d, s_val, ctl, hist2);
        RTOPK_LAUNCH_CHECK();
        k_hist_pass<3><<<grid, kHistThreads, 0, stream>>>(residual, d, s_val, ctl, hist3);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_SELECT, stream);
        const unsigned grid = clamp_grid((L.cap_s + kTileElems - 1) / kTileElems, 1, 1024);
        k_select_top_r<<<grid, kTileThreads, 0, stream>>>(residual, d, s_idx, s_val, ctl, st_gt,
                                                         st_eq, cand_idx, cand_val, r);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_SAMPLE, stream);
        const unsigned grid = clamp_grid((r + 2047) / 2048, 1, 512);
        k_key_hist<<<grid, kHistThreads, 0, stream>>>(cand_idx, r, k, ps, ctl, histk);
        RTOPK_LAUNCH_CHECK();
        k_key_collect<<<grid, kHistThreads, 0, stream>>>(cand_idx, r, ps, ctl, m_key, m_idx);
        RTOPK_LAUNCH_CHECK();
    }
    {
        StageScope sc(trace, RTOPK_STAGE_EMIT, stream);
        k_emit<<<L.tiles_cand, kTileThreads, 0, stream>>>(cand_idx, cand_val, r, k, ps, ctl,
                                                          st_emit, out_idx, out_val, residual);
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
    host_out->path = c.mode;
    host_out->threshold_bits = c.threshold;
    host_out->reserved = 0;
    host_out->count_greater = c.count_greater;
    host_out->ties_taken = c.ties;
    host_out->superset_size = c.mode == kModeSuperset ? c.superset : 0;
    host_out->key_bucket_size = c.key_list;
    return RTOPK_OK;
}
