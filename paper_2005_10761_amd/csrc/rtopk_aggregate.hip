// rtopk_aggregate: the master step of Algorithm 1, ghat = (1/n) sum_i ghat_i,
// from n sorted sparse messages to one dense vector, in a single kernel.
//
// The output is cut into tiles of 2048 consecutive coordinates and every
// WAVEFRONT owns a run of consecutive tiles and an LDS copy of the tile it is
// working on; wavefronts never synchronise with each other. Lane w remembers
// how far the wavefront has come in worker w's ascending index list: where
// the wavefront's first tile starts in it is found once, by a search in which
// the 64 lanes probe several positions per worker at a time. For every tile
// and worker the wavefront then reads the next 64 (index, value) pairs of the
// message with one coalesced load (eight workers' loads in flight together),
// adds the pairs that fall below the tile's end into the LDS tile and moves
// the worker's position on by their number; when a slice fills all 64 lanes
// (the message is crowded in this tile: the top coordinates of one layer) the
// next eight groups of 64 are fetched together and added in order. No search
// is needed from tile to tile.
// Workers are taken in order 0, 1, ... and a wavefront's LDS accesses execute
// in program order, so the order of the binary32 additions is fixed: +0, then
// worker 0, 1, ... The tile is finally divided by n and written with 16-byte
// stores. HBM traffic: 4d bytes written + 8nk bytes read; no atomics, no
// sort, no workspace.
//
// rtopk_aggregate_update applies the master's next line, omega <- omega -
// eta * ghat, to the weights directly, so the dense ghat is never stored and
// only weights that some worker sent are read and written. It uses the same
// 2048-coordinate tiles with one wavefront per tile, but where a tile starts
// in each worker's list is not searched: a first kernel looks at every pair
// of neighbouring entries and, wherever the tile number changes, writes the
// entry's position into a [tile][worker] table for all tiles in between.
// The second kernel reads its tile's row and the next one, leaves at once if
// the tile is empty, and otherwise adds the entries into its LDS tile in
// worker order, then updates the weights at the non-zero positions. With up
// to 16 workers and up to 64 entries per worker in the tile, every entry
// stays in a register of one lane from the load to the store: the weight at
// its index is fetched while the LDS sums are formed, and the first entry to
// swap the finished sum out of LDS writes the new weight.
#include "rtopk_common.h"
#include "../../include/rtopk.h"

#include <mutex>

namespace rtopk {

constexpr int kAggThreads = 256;
constexpr int kAggWaves = kAggThreads / kWave;
constexpr int kAggTile = 2048;
constexpr int kAggAhead = 8;              // workers whose next pairs are fetched together
constexpr int kAggMore = 8;               // further slices of one crowded message fetched together
constexpr unsigned kAggMaxWaves = 4096;
constexpr unsigned kMomentumLdsClaim = 30u * 1024u;   // with the 32 KB of tiles: two workgroups per unit

__device__ __forceinline__ u32 popc_mask(u64 m) { return (u32)__popcll((unsigned long long)m); }

__device__ __forceinline__ u64 read_lane_u64(u64 v, int lane)
{
    const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)v, lane);
    const u32 hi = (u32)__builtin_amdgcn_readlane((int)(u32)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

// For each of nw <= 64 workers (worker w0 + w <-> the group of P lanes
// starting at lane w * P, P = the largest power of two with nw * P <= 64): the
// first position in the worker's ascending index list whose entry is >= x.
// Every step the P lanes of a group probe P evenly spaced positions of the
// remaining range, which shrinks (P + 1)-fold. Returns the result of worker
// `lane` in lane `lane` (lanes >= nw: unspecified).
__device__ __forceinline__ u64 wave_lower_bounds(const u32 *__restrict__ idx, u32 w0, u32 nw, u64 k,
                                                 u64 x)
{
    const u32 lane = lane_id();
    u32 P = 1;
    while (2 * P * nw <= (u32)kWave) P *= 2;
    const u32 w = lane / P, p = lane % P;
    const bool live = w < nw;
    const u32 *wi = idx + (u64)(w0 + (live ? w : 0)) * k;
    u64 lo = 0, hi = live ? k : 0;                  // the answer lies in [lo, hi]
    const float inv = 1.0f / (float)(P + 1);
    while (__any(hi > lo)) {
        // probe positions lo <= pos_0 <= pos_1 <= ... < hi, roughly evenly spaced (any
        // non-decreasing choice inside the range is valid; this one needs no division)
        const float len = (float)(hi - lo);
        auto probe_at = [&](u32 q) {
            const u64 t = lo + (u64)(len * ((float)(q + 1) * inv));
            return t < hi ? t : hi - 1;
        };
        const bool below = hi > lo && (u64)wi[probe_at(p)] < x;
        const u64 mask = __ballot(below);
        // sorted list: the group's probes below x form a prefix
        const u32 m = __popcll((mask >> (w * P)) & (P == 64 ? ~0ull : ((1ull << P) - 1ull)));
        if (hi > lo) {
            const u64 new_lo = m > 0 ? probe_at(m - 1) + 1 : lo;
            const u64 new_hi = m < P ? probe_at(m) : hi;
            lo = new_lo;
            hi = new_hi;
        }
    }
    // hand the result of worker w (held by all lanes of group w) to lane w
    const u32 lo_lo = __shfl((u32)lo, (int)((lane < nw ? lane : 0) * P), kWave);
    const u32 lo_hi = __shfl((u32)(lo >> 32), (int)((lane < nw ? lane : 0) * P), kWave);
    return ((u64)lo_hi << 32) | lo_lo;
}

// What the momentum form of the kernel does with the average of a coordinate:
// u = scale * average, v <- fma(mu, v, u), w <- fma(neg_eta, v, w) with the
// rounded new velocity.
struct Momentum {
    float scale, mu, neg_eta;
    float *velocity;
};

// kMomentum == false: out[i] = average[i].
// kMomentum == true:  out is the weight vector w; see Momentum.
template <bool kMomentum>
__global__ void __launch_bounds__(kAggThreads)
k_aggregate(const u32 *__restrict__ idx, const float *__restrict__ val, u32 n, u64 k, u64 d,
            u64 tiles, u32 tiles_per_wave, float *__restrict__ out, Momentum mom)
{
    __shared__ float tile_s[kAggWaves][kAggTile];
    const u32 lane = lane_id(), wave = threadIdx.x / kWave;
    float *tile = tile_s[wave];
    const u64 gw = (u64)blockIdx.x * kAggWaves + wave;
    const u64 first_tile = gw * tiles_per_wave;
    const u64 last_tile = first_tile + tiles_per_wave < tiles ? first_tile + tiles_per_wave : tiles;
    if (first_tile >= last_tile) return;
    // one correctly rounded division per output; for n a power of two the
    // product with 1/n is the same number
    const float fn = (float)n;
    const bool n_pow2 = (n & (n - 1u)) == 0u;
    const float rn = 1.0f / fn;
    const bool out_vec =
        (((uintptr_t)out | (kMomentum ? (uintptr_t)mom.velocity : (uintptr_t)0)) & 15u) == 0;
    auto step = [&](float avg, float &v, float &w) {
        const float u = mom.scale * avg;
        v = fmaf(mom.mu, v, u);
        w = fmaf(mom.neg_eta, v, w);
    };
    const u32 groups = (n + kWave - 1) / kWave;    // workers are taken 64 at a time
    // lane w: where the current tile starts in the message of worker w (first group only;
    // with more than 64 workers the position is searched again for every tile)
    u64 pos0 = 0;
    if (groups == 1) pos0 = wave_lower_bounds(idx, 0, n, k, first_tile * kAggTile);

    for (u64 t = first_tile; t < last_tile; ++t) {
        const u64 tile_base = t * kAggTile;
        const u64 tile_end = tile_base + kAggTile < d ? tile_base + kAggTile : d;
        for (int i = lane; i < kAggTile / 4; i += kWave)
            reinterpret_cast<float4 *>(tile)[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

        for (u32 w0 = 0; w0 < n; w0 += kWave) {
            const u32 nw = n - w0 < (u32)kWave ? n - w0 : (u32)kWave;
            u64 lo = groups == 1 ? pos0 : wave_lower_bounds(idx, w0, nw, k, tile_base);
            // ---- worker after worker: the next 64 pairs of its message in one
            //      coalesced load, those below the tile's end added into the tile;
            //      the loads of kAggAhead workers are in flight together --------
            for (u32 g0 = 0; g0 < nw; g0 += kAggAhead) {
                u64 from[kAggAhead];
                u32 ri[kAggAhead];
                float rv[kAggAhead];
#pragma unroll
                for (int q = 0; q < kAggAhead; ++q) {
                    const u32 w = g0 + q < nw ? g0 + q : nw - 1;
                    from[q] = read_lane_u64(lo, (int)w);
                    const u64 j = from[q] + lane;
                    const bool in = g0 + q < nw && j < k;
                    ri[q] = in ? idx[(u64)(w0 + w) * k + j] : 0xFFFFFFFFu;
                    rv[q] = in ? val[(u64)(w0 + w) * k + j] : 0.0f;
                }
#pragma unroll
                for (int q = 0; q < kAggAhead; ++q) {
                    if (g0 + q >= nw) break;
                    const u32 w = g0 + q;
                    const u32 *si = idx + (u64)(w0 + w) * k;
                    const float *sv = val + (u64)(w0 + w) * k;
                    u64 at = from[q];
                    // 64 pairs into the tile; returns how many of them lay inside it
                    auto add_slice = [&](u32 i, float v) -> u32 {
                        const bool inside = (u64)i < tile_end;     // 0xFFFFFFFF marks "no entry"
                        const u64 mask = __ballot(inside);         // a prefix of the lanes: sorted
                        // repeated indices inside one message (never produced by the
                        // encoder, but allowed) must be added in position order
                        const u32 left = __shfl_up(i, 1, kWave);
                        const bool dup = inside && lane > 0 && left == i;
                        if (!__any(dup)) {
                            if (inside) tile[i - tile_base] += v;
                        } else {
                            for (u64 rest = mask; rest; rest &= rest - 1) {
                                const int src = __ffsll((unsigned long long)rest) - 1;
                                if ((int)lane == src) tile[i - tile_base] += v;
                            }
                        }
                        return popc_mask(mask);
                    };
                    u32 took = add_slice(ri[q], rv[q]);
                    at += took;
                    // The slice filled all 64 lanes: the message is crowded here (its
                    // entries cluster in a few tiles). The next kAggMore slices are
                    // fetched together and added in order up to the first that ends
                    // inside the tile.
                    while (took == (u32)kWave) {
                        u32 mi[kAggMore];
                        float mv[kAggMore];
#pragma unroll
                        for (int s2 = 0; s2 < kAggMore; ++s2) {
                            const u64 j = at + (u64)s2 * kWave + lane;
                            mi[s2] = j < k ? si[j] : 0xFFFFFFFFu;
                            mv[s2] = j < k ? sv[j] : 0.0f;
                        }
#pragma unroll
                        for (int s2 = 0; s2 < kAggMore; ++s2) {
                            if (took == (u32)kWave) {
                                took = add_slice(mi[s2], mv[s2]);
                                at += took;
                            }
                        }
                    }
                    // the new position of worker w goes back into lane w
                    if (lane == w) lo = at;
                }
            }
            if (groups == 1) pos0 = lo;
        }
        if (out_vec && tile_base + kAggTile <= d) {
            float4 *o4 = reinterpret_cast<float4 *>(out + tile_base);
            constexpr int kVecs = kAggTile / 4 / kWave;
            // weights and velocity are read once and written once, in place: both
            // carry the streaming hint (as in the encoder's streaming kernel, where
            // the hint on load and store together is worth 15%)
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            f32x4 vel[kMomentum ? kVecs : 1], wgt[kMomentum ? kVecs : 1];
            f32x4 *v4 = nullptr, *w4 = reinterpret_cast<f32x4 *>(o4);
            if (kMomentum) {
                v4 = reinterpret_cast<f32x4 *>(mom.velocity + tile_base);
#pragma unroll
                for (int q = 0; q < kVecs; ++q) {
                    vel[q] = __builtin_nontemporal_load(v4 + q * kWave + lane);
                    wgt[q] = __builtin_nontemporal_load(w4 + q * kWave + lane);
                }
            }
#pragma unroll
            for (int q = 0; q < kVecs; ++q) {
                const int i = q * kWave + lane;
                float4 v = reinterpret_cast<const float4 *>(tile)[i];
                if (n_pow2) { v.x *= rn; v.y *= rn; v.z *= rn; v.w *= rn; }
                else { v.x /= fn; v.y /= fn; v.z /= fn; v.w /= fn; }
                if (kMomentum) {
                    const int m = kMomentum ? q : 0;
                    const float avg[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        float ve = vel[m][c], we = wgt[m][c];
                        step(avg[c], ve, we);
                        vel[m][c] = ve;
                        wgt[m][c] = we;
                    }
                    __builtin_nontemporal_store(vel[m], v4 + i);
                    __builtin_nontemporal_store(wgt[m], w4 + i);
                } else {
                    o4[i] = v;
                }
            }
        } else {
            for (u64 i = lane; tile_base + i < tile_end; i += kWave) {
                const float avg = tile[i] / fn;
                if (kMomentum) {
                    float v = mom.velocity[tile_base + i], w = out[tile_base + i];
                    step(avg, v, w);
                    mom.velocity[tile_base + i] = v;
                    out[tile_base + i] = w;
                } else {
                    out[tile_base + i] = avg;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// tile_starts: start[t * n + w] = the first position in worker w's list whose
// index lies in tile t or later, for t = 0 .. tiles (the last row is k).
// Thread j of worker w compares the tiles of entries j - 1 and j (tile -1
// before the list, tile `tiles` after it) and fills the rows in between;
// since the list ascends, every row is written exactly once. A long run of
// empty tiles is filled by the whole wavefront. blockIdx.y is the worker.
// ---------------------------------------------------------------------------
constexpr int kStartThreads = 256;

__global__ void __launch_bounds__(kStartThreads)
k_tile_starts(const u32 *__restrict__ idx, u32 n, u64 k, u64 tiles, u32 *__restrict__ start)
{
    const u32 w = blockIdx.y;
    const u32 *wi = idx + (u64)w * k;
    const u64 j = (u64)blockIdx.x * kStartThreads + threadIdx.x;
    // rows (from, to] get the value j; an index past the last tile (a broken
    // precondition) is treated as the end of the list
    u64 from = 0, to = 0;
    if (j <= k) {
        const u64 t_prev = j > 0 ? (u64)wi[j - 1] / kAggTile + 1 : 0;   // first row to fill
        u64 t_cur = j < k ? (u64)wi[j] / kAggTile : tiles;
        if (t_cur > tiles) t_cur = tiles;
        from = t_prev;
        to = t_cur + 1;                                                  // one past the last row
        if (to < from) to = from;
    }
    const bool is_long = to - from > 8;
    if (!is_long)
        for (u64 t = from; t < to; ++t) start[t * n + w] = (u32)j;
    for (u64 rest = __ballot(is_long); rest; rest &= rest - 1) {
        const int src = __ffsll((unsigned long long)rest) - 1;
        const u64 a = read_lane_u64(from, src), b = read_lane_u64(to, src);
        const u32 v = (u32)read_lane_u64(j, src);
        for (u64 t = a + lane_id(); t < b; t += kWave) start[t * n + w] = v;
    }
}

// ---------------------------------------------------------------------------
// update: one wavefront per tile. omega[i] = fma(neg_step, average[i],
// omega[i]) wherever the average of what the workers sent for i is not zero.
// ---------------------------------------------------------------------------
constexpr u32 kDenseTileEntries = 512;     // from here on the whole tile is read and written
constexpr int kUpdateAhead = 16;           // workers whose entries are held in registers together

__global__ void __launch_bounds__(kAggThreads)
k_update(const u32 *__restrict__ idx, const float *__restrict__ val, u32 n, u64 k, u64 d,
         u64 tiles, const u32 *__restrict__ start, float neg_step, float *__restrict__ omega)
{
    __shared__ float tile_s[kAggWaves][kAggTile];
    const u32 lane = lane_id(), wave = threadIdx.x / kWave;
    float *tile = tile_s[wave];
    const u64 t = (u64)blockIdx.x * kAggWaves + wave;
    if (t >= tiles) return;
    const u64 tile_base = t * kAggTile;
    const u64 tile_end = tile_base + kAggTile < d ? tile_base + kAggTile : d;
    const float fn = (float)n;
    const bool n_pow2 = (n & (n - 1u)) == 0u;
    const float rn = 1.0f / fn;
    bool cleared = false;
    u32 entries = 0;
    // the average of a coordinate from its sum; a weight moves only where the
    // AVERAGE is not zero (a tiny sum may underflow in the division)
    auto average = [&](float sum) { return n_pow2 ? sum * rn : sum / fn; };
    auto step = [&](float avg, float w) { return fmaf(neg_step, avg, w); };

    // ---- few workers with at most 64 entries each in this tile (the usual
    //      case): every entry stays in a register of "its" lane. The weight at
    //      the entry's index is fetched while the sums are formed in LDS;
    //      afterwards every entry swaps a zero into its LDS word, and the one
    //      that gets the sum back (the first to arrive) writes the weight. ----
    if (n <= kUpdateAhead) {
        u32 lo = 0, cnt = 0;
        if (lane < n) {
            u64 a = start[t * n + lane], b = start[(t + 1) * n + lane];
            if (b > k) b = k;
            if (a > b) a = b;
            lo = (u32)a;
            cnt = (u32)(b - a);
        }
        if (__ballot(cnt != 0u) == 0ull) return;           // nobody sent anything in this tile
        if (__ballot(cnt > (u32)kWave) == 0ull) {
            for (int i = lane; i < kAggTile / 4; i += kWave)
                reinterpret_cast<float4 *>(tile)[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            u32 ei[kUpdateAhead];
            float ev[kUpdateAhead], ew[kUpdateAhead];
            bool in[kUpdateAhead];
#pragma unroll
            for (int q = 0; q < kUpdateAhead; ++q) {
                in[q] = false;
                ei[q] = 0xFFFFFFFFu;
                ev[q] = 0.0f;
                if ((u32)q < n) {
                    const u32 from = (u32)__builtin_amdgcn_readlane((int)lo, q);
                    const u32 c = (u32)__builtin_amdgcn_readlane((int)cnt, q);
                    if (lane < c) {
                        ei[q] = idx[(u64)q * k + from + lane];
                        ev[q] = val[(u64)q * k + from + lane];
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < kUpdateAhead; ++q) {
                // the range check keeps a list that is not sorted (a broken
                // precondition) inside the LDS tile
                in[q] = (u64)ei[q] >= tile_base && (u64)ei[q] < tile_end;
                ew[q] = in[q] ? omega[ei[q]] : 0.0f;
            }
#pragma unroll
            for (int q = 0; q < kUpdateAhead; ++q) {
                if ((u32)q < n) {
                    // repeated indices inside one message must be added in position order
                    const u32 mine = ei[q];
                    const float v = ev[q];
                    const bool inside = in[q];
                    const u32 left = __shfl_up(mine, 1, kWave);
                    const bool dup = inside && lane > 0 && left == mine;
                    if (!__any(dup)) {
                        if (inside) tile[mine - tile_base] += v;
                    } else {
                        for (u64 rest = __ballot(inside); rest; rest &= rest - 1) {
                            const int src = __ffsll((unsigned long long)rest) - 1;
                            if ((int)lane == src) tile[mine - tile_base] += v;
                        }
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < kUpdateAhead; ++q) {
                if ((u32)q < n && in[q]) {
                    const float avg = average(atomicExch(&tile[ei[q] - tile_base], 0.0f));
                    if (avg != 0.0f) omega[ei[q]] = step(avg, ew[q]);
                }
            }
            return;
        }
    }

    for (u32 w0 = 0; w0 < n; w0 += kWave) {
        const u32 nw = n - w0 < (u32)kWave ? n - w0 : (u32)kWave;
        // lane w: the part [lo, hi) of worker w0 + w's list that lies in this tile
        u64 lo = 0, hi = 0;
        if (lane < nw) {
            lo = start[t * n + w0 + lane];
            hi = start[(t + 1) * n + w0 + lane];
            if (hi > k) hi = k;
            if (lo > hi) lo = hi;
        }
        const u32 here = wave_sum((u32)(hi - lo));
        if (here == 0u) continue;
        if (!cleared) {
            for (int i = lane; i < kAggTile / 4; i += kWave)
                reinterpret_cast<float4 *>(tile)[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            cleared = true;
        }
        entries += here;
        for (u32 g0 = 0; g0 < nw; g0 += kAggAhead) {
            u64 from[kAggAhead], to[kAggAhead];
            u32 ri[kAggAhead];
            float rv[kAggAhead];
#pragma unroll
            for (int q = 0; q < kAggAhead; ++q) {
                const u32 w = g0 + q < nw ? g0 + q : nw - 1;
                from[q] = read_lane_u64(lo, (int)w);
                to[q] = g0 + q < nw ? read_lane_u64(hi, (int)w) : from[q];
                const u64 j = from[q] + lane;
                const bool in = j < to[q];
                ri[q] = in ? idx[(u64)(w0 + w) * k + j] : 0xFFFFFFFFu;
                rv[q] = in ? val[(u64)(w0 + w) * k + j] : 0.0f;
            }
#pragma unroll
            for (int q = 0; q < kAggAhead; ++q) {
                if (g0 + q >= nw) break;
                const u32 *si = idx + (u64)(w0 + g0 + q) * k;
                const float *sv = val + (u64)(w0 + g0 + q) * k;
                u64 at = from[q];
                u32 i = ri[q];
                float v = rv[q];
                while (at < to[q]) {
                    // the table says these entries belong to the tile; the check keeps a
                    // list that is not sorted (a broken precondition) inside the LDS tile
                    const bool inside = at + lane < to[q] && (u64)i >= tile_base && (u64)i < tile_end;
                    // repeated indices inside one message must be added in position order
                    const u32 left = __shfl_up(i, 1, kWave);
                    const bool dup = inside && lane > 0 && left == i;
                    if (!__any(dup)) {
                        if (inside) tile[i - tile_base] += v;
                    } else {
                        for (u64 rest = __ballot(inside); rest; rest &= rest - 1) {
                            const int src = __ffsll((unsigned long long)rest) - 1;
                            if ((int)lane == src) tile[i - tile_base] += v;
                        }
                    }
                    at += kWave;
                    if (at >= to[q]) break;
                    const u64 j = at + lane;
                    i = j < to[q] ? si[j] : 0xFFFFFFFFu;
                    v = j < to[q] ? sv[j] : 0.0f;
                }
            }
        }
    }
    if (!cleared) return;                               // nobody sent anything in this tile

    constexpr int kVecs = kAggTile / 4 / kWave;         // float4 per lane
    float4 s4[kVecs];                                   // the averages of this lane's coordinates
#pragma unroll
    for (int q = 0; q < kVecs; ++q) {
        const float4 t4 = reinterpret_cast<const float4 *>(tile)[q * kWave + lane];
        s4[q] = make_float4(average(t4.x), average(t4.y), average(t4.z), average(t4.w));
    }
    if (entries >= kDenseTileEntries && ((uintptr_t)omega & 15u) == 0 &&
        tile_base + kAggTile <= d) {
        float4 *o4 = reinterpret_cast<float4 *>(omega + tile_base);
        float4 w[kVecs];
#pragma unroll
        for (int q = 0; q < kVecs; ++q) w[q] = o4[q * kWave + lane];
#pragma unroll
        for (int q = 0; q < kVecs; ++q) {
            const float4 s = s4[q];
            if (s.x == 0.0f && s.y == 0.0f && s.z == 0.0f && s.w == 0.0f) continue;
            if (s.x != 0.0f) w[q].x = step(s.x, w[q].x);
            if (s.y != 0.0f) w[q].y = step(s.y, w[q].y);
            if (s.z != 0.0f) w[q].z = step(s.z, w[q].z);
            if (s.w != 0.0f) w[q].w = step(s.w, w[q].w);
            o4[q * kWave + lane] = w[q];
        }
    } else {
        // few entries: only the weights that move are read; all loads first
        float *o = omega + tile_base + 4 * lane;
        float w[kVecs][4];
#pragma unroll
        for (int q = 0; q < kVecs; ++q) {
            const float sv[4] = {s4[q].x, s4[q].y, s4[q].z, s4[q].w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                w[q][c] = sv[c] != 0.0f ? o[q * 4 * kWave + c] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < kVecs; ++q) {
            const float sv[4] = {s4[q].x, s4[q].y, s4[q].z, s4[q].w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (sv[c] != 0.0f) o[q * 4 * kWave + c] = step(sv[c], w[q][c]);
        }
    }
}

#ifdef RTOPK_DEBUG_CHECKS
// ---------------------------------------------------------------------------
// Debug build only: the preconditions of the master entry points (every index
// below d, every worker's slice ascending) are checked on the device before
// the call's own kernels are enqueued. The check synchronises the stream, so
// it is kept out of the release build, where the conditions stay preconditions.
// ---------------------------------------------------------------------------
static __device__ u32 dbg_bad_entries;

__global__ void k_check_messages(const u32 *__restrict__ idx, u32 n, u64 k, u64 d, u32 *bad)
{
    const u64 total = (u64)n * k;
    u32 mine = 0;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (u64)gridDim.x * blockDim.x) {
        const u32 v = idx[i];
        if ((u64)v >= d) ++mine;
        else if (i % k != 0 && idx[i - 1] > v) ++mine;
    }
    if (mine) atomicAdd(bad, mine);
}
#endif

}  // namespace rtopk

using namespace rtopk;

// Release build: nothing. Debug build (RTOPK_DEBUG_CHECKS): RTOPK_EINVAL when a
// message breaks a precondition of the master entry points.
static int debug_check_messages(const uint32_t *idx, uint32_t n, uint64_t k, uint64_t d,
                                hipStream_t stream)
{
#ifdef RTOPK_DEBUG_CHECKS
    u32 *bad = nullptr;
    u32 host_bad = 0;
    if (hipGetSymbolAddress((void **)&bad, HIP_SYMBOL(dbg_bad_entries)) != hipSuccess ||
        hipMemcpyAsync(bad, &host_bad, sizeof host_bad, hipMemcpyHostToDevice, stream) != hipSuccess)
        return RTOPK_EHIP;
    k_check_messages<<<1024, 256, 0, stream>>>(idx, n, k, d, bad);
    if (hipGetLastError() != hipSuccess ||
        hipMemcpyAsync(&host_bad, bad, sizeof host_bad, hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return RTOPK_EHIP;
    if (host_bad != 0) return RTOPK_EINVAL;
#else
    (void)idx; (void)n; (void)k; (void)d; (void)stream;
#endif
    return RTOPK_OK;
}

extern "C" int rtopk_aggregate_workspace_bytes(uint64_t d, uint32_t n, uint64_t k,
                                               uint64_t *bytes)
{
    if (!bytes || n < 1 || k < 1 || d < 1 || d > 0xFFFFFFFFull) return RTOPK_EINVAL;
    *bytes = 0;   // the single-kernel aggregator keeps everything in LDS
    return RTOPK_OK;
}

extern "C" int rtopk_aggregate(const uint32_t *idx, const float *val, uint32_t n, uint64_t k,
                               uint64_t d, float *out, void *workspace,
                               uint64_t workspace_bytes, void *stream_v)
{
    (void)workspace_bytes;
    if (!idx || !val || !out || n < 1 || k < 1 || d < 1 || d > 0xFFFFFFFFull)
        return RTOPK_EINVAL;
    if (workspace && ((uintptr_t)workspace & 255u)) return RTOPK_EWORKSPACE;
    hipStream_t stream = (hipStream_t)stream_v;
    if (const int rc = debug_check_messages(idx, n, k, d, stream)) return rc;
    const u64 tiles = (d + kAggTile - 1) / kAggTile;
    const u32 tiles_per_wave = (u32)((tiles + kAggMaxWaves - 1) / kAggMaxWaves);
    const u64 waves = (tiles + tiles_per_wave - 1) / tiles_per_wave;
    const unsigned grid = (unsigned)((waves + kAggWaves - 1) / kAggWaves);
    k_aggregate<false><<<grid, kAggThreads, 0, stream>>>(idx, val, n, k, d, tiles, tiles_per_wave,
                                                         out, Momentum{});
    if (hipGetLastError() != hipSuccess) return RTOPK_EHIP;
    return RTOPK_OK;
}

extern "C" int rtopk_aggregate_update_momentum(const uint32_t *idx, const float *val, uint32_t n,
                                               uint64_t k, uint64_t d, float eta, float scale,
                                               float mu, float *omega, float *velocity,
                                               void *stream_v)
{
    if (!idx || !val || !omega || !velocity || n < 1 || k < 1 || d < 1 || d > 0xFFFFFFFFull)
        return RTOPK_EINVAL;
    {
        const uintptr_t w0 = (uintptr_t)omega, v0 = (uintptr_t)velocity;
        if (w0 < v0 + d * 4 && v0 < w0 + d * 4) return RTOPK_EINVAL;
    }
    hipStream_t stream = (hipStream_t)stream_v;
    if (const int rc = debug_check_messages(idx, n, k, d, stream)) return rc;
    const u64 tiles = (d + kAggTile - 1) / kAggTile;
    const u32 tiles_per_wave = (u32)((tiles + kAggMaxWaves - 1) / kAggMaxWaves);
    const u64 waves = (tiles + tiles_per_wave - 1) / tiles_per_wave;
    const unsigned grid = (unsigned)((waves + kAggWaves - 1) / kAggWaves);
    // This form streams 16 bytes per coordinate and is bound by HBM alone: two
    // workgroups per compute unit (eight wavefronts) stream 6% faster than the five
    // that fit, so each workgroup also claims LDS it does not use.
    k_aggregate<true><<<grid, kAggThreads, kMomentumLdsClaim, stream>>>(
        idx, val, n, k, d, tiles, tiles_per_wave, omega, Momentum{scale, mu, -eta, velocity});
    if (hipGetLastError() != hipSuccess) return RTOPK_EHIP;
    return RTOPK_OK;
}

extern "C" int rtopk_aggregate_update_workspace_bytes(uint64_t d, uint32_t n, uint64_t k,
                                                      uint64_t *bytes)
{
    if (!bytes || n < 1 || k < 1 || k > 0xFFFFFFFFull || d < 1 || d > 0xFFFFFFFFull)
        return RTOPK_EINVAL;
    const u64 tiles = (d + kAggTile - 1) / kAggTile;
    *bytes = align_up((tiles + 1) * (u64)n * sizeof(u32), 256);
    return RTOPK_OK;
}

// the two kernels of the fused update; `start` holds (tiles + 1) * n words
static int launch_update(const uint32_t *idx, const float *val, uint32_t n, uint64_t k, uint64_t d,
                         float eta, float scale, float *omega, u32 *start, hipStream_t stream)
{
    if (const int rc = debug_check_messages(idx, n, k, d, stream)) return rc;
    const u64 tiles = (d + kAggTile - 1) / kAggTile;
    const dim3 sgrid((unsigned)((k + 1 + kStartThreads - 1) / kStartThreads), n);
    k_tile_starts<<<sgrid, kStartThreads, 0, stream>>>(idx, n, k, tiles, start);
    if (hipGetLastError() != hipSuccess) return RTOPK_EHIP;
    volatile float step = eta * scale;                  // one binary32 rounding, then negated
    const unsigned grid = (unsigned)((tiles + kAggWaves - 1) / kAggWaves);
    k_update<<<grid, kAggThreads, 0, stream>>>(idx, val, n, k, d, tiles, start, -step, omega);
    if (hipGetLastError() != hipSuccess) return RTOPK_EHIP;
    return RTOPK_OK;
}

extern "C" int rtopk_aggregate_update(const uint32_t *idx, const float *val, uint32_t n,
                                      uint64_t k, uint64_t d, float eta, float scale,
                                      float *omega, void *workspace, uint64_t workspace_bytes,
                                      void *stream_v)
{
    uint64_t need = 0;
    if (!idx || !val || !omega || rtopk_aggregate_update_workspace_bytes(d, n, k, &need) != RTOPK_OK)
        return RTOPK_EINVAL;
    if (n > 65535u) return RTOPK_EINVAL;                // workers are a grid dimension
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < need)
        return RTOPK_EWORKSPACE;
    return launch_update(idx, val, n, k, d, eta, scale, omega, static_cast<u32 *>(workspace),
                         (hipStream_t)stream_v);
}

// ---------------------------------------------------------------------------
// rtopk_aggregate_update_static: the same two kernels with the tile-start
// table in a device array that is part of the library's code object, for
// callers that can neither allocate nor pass a workspace. Every device the
// library runs on holds its own copy of the array at its own address; the
// address is looked up once per device, with that device current, and kept.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[RTOPK_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxScratchDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxScratchDevices];      // device address of `scratch`, per device

int static_scratch(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return RTOPK_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        // in host code the array's name is only a handle: the device address comes from here
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RTOPK_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RTOPK_OK;
}
}  // namespace

extern "C" int rtopk_aggregate_update_static(const uint32_t *idx, const float *val, uint32_t n,
                                             uint64_t k, uint64_t d, float eta, float scale,
                                             float *omega, void *stream_v)
{
    uint64_t need = 0;
    if (!idx || !val || !omega || rtopk_aggregate_update_workspace_bytes(d, n, k, &need) != RTOPK_OK)
        return RTOPK_EINVAL;
    if (n > 65535u) return RTOPK_EINVAL;
    if (need > (uint64_t)RTOPK_STATIC_SCRATCH_BYTES) return RTOPK_ETOOLARGE;
    void *table = nullptr;
    const int rc = static_scratch(&table);
    if (rc) return rc;
    // k_tile_starts writes every word of the table that k_update reads, so
    // nothing of what the previous call left in the array has to be cleared
    return launch_update(idx, val, n, k, d, eta, scale, omega, static_cast<u32 *>(table),
                         (hipStream_t)stream_v);
}

extern "C" const char *rtopk_strerror(int code)
{
    switch (code) {
    case RTOPK_OK: return "ok";
    case RTOPK_EINVAL: return "invalid argument (null pointer, sizes outside 1 <= k <= r <= d < 2^32, n < 1, or grad overlaps residual)";
    case RTOPK_EWORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case RTOPK_EHIP: return "a HIP call or kernel launch failed";
    case RTOPK_ETOOLARGE: return "sizes exceed the library's built-in scratch array (rtopk_aggregate_update_static needs 4 bytes per worker and per 2048 coordinates within RTOPK_STATIC_SCRATCH_BYTES); use the entry point that takes a workspace";
    default: return "unknown rtopk error code";
    }
}

extern "C" int rtopk_version(void) { return 200; }

// 1 when the library was built with RTOPK_DEBUG_CHECKS, else 0
extern "C" int rtopk_debug_checks(void)
{
#ifdef RTOPK_DEBUG_CHECKS
    return 1;
#else
    return 0;
#endif
}
