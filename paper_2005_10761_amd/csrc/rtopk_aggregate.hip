// rtopk_aggregate: the master step of Algorithm 1, ghat = (1/n) sum_i ghat_i,
// from n sorted sparse messages to one dense vector, in a single kernel.
//
// Each workgroup owns one tile of 4096 consecutive output coordinates. For
// every worker it finds, by binary search in that worker's ascending index
// list, the slice of the message that falls into the tile, and adds the
// slice into an LDS copy of the tile, one worker after the other (so the
// order of the binary32 additions is fixed: +0, then worker 0, 1, ...). The
// tile is then divided by n and written with 16-byte stores. HBM traffic:
// 4d bytes written + 8nk bytes read; no global atomics, no sort.
#include "rtopk_common.h"
#include "../../include/rtopk.h"

namespace rtopk {

constexpr int kAggThreads = 256;
constexpr int kAggTile = 4096;
constexpr int kAggWorkerChunk = 64;

__device__ __forceinline__ u64 lower_bound_u32(const u32 *__restrict__ a, u64 n, u64 x)
{
    u64 lo = 0, hi = n;
    while (lo < hi) {
        const u64 mid = (lo + hi) >> 1;
        if ((u64)a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ void __launch_bounds__(kAggThreads)
k_aggregate(const u32 *__restrict__ idx, const float *__restrict__ val, u32 n, u64 k, u64 d,
            float *__restrict__ out)
{
    __shared__ float tile[kAggTile];
    __shared__ u64 lo_s[kAggWorkerChunk], hi_s[kAggWorkerChunk];
    const u64 tile_base = (u64)blockIdx.x * kAggTile;
    const u64 tile_end = tile_base + kAggTile < d ? tile_base + kAggTile : d;
    for (int t = threadIdx.x; t < kAggTile; t += kAggThreads) tile[t] = 0.0f;

    for (u32 w0 = 0; w0 < n; w0 += kAggWorkerChunk) {
        const u32 nw = n - w0 < (u32)kAggWorkerChunk ? n - w0 : (u32)kAggWorkerChunk;
        __syncthreads();
        if (threadIdx.x < 2 * nw) {
            const u32 w = threadIdx.x >> 1;
            const u32 *wi = idx + (u64)(w0 + w) * k;
            if (threadIdx.x & 1) hi_s[w] = lower_bound_u32(wi, k, tile_end);
            else lo_s[w] = lower_bound_u32(wi, k, tile_base);
        }
        __syncthreads();
        for (u32 w = 0; w < nw; ++w) {
            const u64 b = lo_s[w], e = hi_s[w];
            const u32 *wi = idx + (u64)(w0 + w) * k;
            const float *wv = val + (u64)(w0 + w) * k;
            for (u64 j = b + threadIdx.x; j < e; j += kAggThreads) {
                const u32 i = wi[j];
                // a repeated index is folded in by the first entry of its run
                if (j > b && wi[j - 1] == i) continue;
                float s = tile[i - tile_base];
                u64 jj = j;
                do { s += wv[jj]; ++jj; } while (jj < e && wi[jj] == i);
                tile[i - tile_base] = s;
            }
            __syncthreads();
        }
    }
    __syncthreads();
    const float fn = (float)n;
    const bool vec_ok = ((uintptr_t)out & 15u) == 0 && tile_base + kAggTile <= d;
    if (vec_ok) {
        float4 *o4 = reinterpret_cast<float4 *>(out + tile_base);
        for (int t = threadIdx.x; t < kAggTile / 4; t += kAggThreads) {
            float4 v;
            v.x = tile[4 * t + 0] / fn; v.y = tile[4 * t + 1] / fn;
            v.z = tile[4 * t + 2] / fn; v.w = tile[4 * t + 3] / fn;
            o4[t] = v;
        }
    } else {
        for (u64 t = threadIdx.x; tile_base + t < tile_end; t += kAggThreads)
            out[tile_base + t] = tile[t] / fn;
    }
}

}  // namespace rtopk

using namespace rtopk;

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
    const u64 tiles = (d + kAggTile - 1) / kAggTile;
    k_aggregate<<<(unsigned)tiles, kAggThreads, 0, stream>>>(idx, val, n, k, d, out);
    if (hipGetLastError() != hipSuccess) return RTOPK_EHIP;
    return RTOPK_OK;
}

extern "C" const char *rtopk_strerror(int code)
{
    switch (code) {
    case RTOPK_OK: return "ok";
    case RTOPK_EINVAL: return "invalid argument (null pointer, sizes outside 1 <= k <= r <= d < 2^32, n < 1, or grad overlaps residual)";
    case RTOPK_EWORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case RTOPK_EHIP: return "a HIP call or kernel launch failed";
    default: return "unknown rtopk error code";
    }
}

extern "C" int rtopk_version(void) { return 100; }
