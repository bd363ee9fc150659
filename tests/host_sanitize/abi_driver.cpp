// Host-side exercise of the rTop-k library for the sanitizer build: the two
// .hip sources are compiled into this program with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code, and every path that runs
// without launching a kernel is called: workspace sizing over many sizes (the
// chunk geometry, the key window and the workspace layout are computed on the
// host), every argument check of every entry point, the error strings.
// No GPU is needed: every call here returns before its first launch.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/rtopk.h"
#include "../../include/rtopk_diag.h"

static int failures = 0;
#define EXPECT(cond)                                                         \
    do {                                                                     \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
    } while (0)

int main()
{
    // ---- sizing: the domain of Definition 3 and a sweep of legal sizes -----
    uint64_t bytes = 0;
    EXPECT(rtopk_encode_workspace_bytes(10, 5, 0, &bytes) == RTOPK_EINVAL);
    EXPECT(rtopk_encode_workspace_bytes(10, 5, 6, &bytes) == RTOPK_EINVAL);
    EXPECT(rtopk_encode_workspace_bytes(10, 11, 5, &bytes) == RTOPK_EINVAL);
    EXPECT(rtopk_encode_workspace_bytes(1ull << 32, 5, 5, &bytes) == RTOPK_EINVAL);
    EXPECT(rtopk_encode_workspace_bytes(10, 5, 5, nullptr) == RTOPK_EINVAL);
    const uint64_t ds[] = {1, 2, 3, 63, 64, 255, 1023, 1024, 1025, 4096, 100003, 1u << 20,
                           11173962, 25557032, 66034000, 1u << 28, 0xFFFFFFFFull};
    uint64_t checksum = 0;
    for (uint64_t d : ds) {
        const uint64_t rs[] = {1, d / 1000 + 1, d / 100 + 1, d / 2 + 1, d};
        for (uint64_t r : rs) {
            if (r > d) continue;
            const uint64_t ks[] = {1, r / 10 + 1, r / 2 + 1, r};
            for (uint64_t k : ks) {
                if (k > r) continue;
                bytes = 0;
                EXPECT(rtopk_encode_workspace_bytes(d, r, k, &bytes) == RTOPK_OK);
                EXPECT(bytes > 0 && bytes % 256 == 0);
                checksum += bytes;
            }
        }
        for (uint32_t n : {1u, 3u, 16u, 65535u}) {
            uint64_t a = 1, b = 0;
            EXPECT(rtopk_aggregate_workspace_bytes(d, n, 1, &a) == RTOPK_OK);
            EXPECT(rtopk_aggregate_update_workspace_bytes(d, n, 1, &b) == RTOPK_OK && b % 256 == 0);
            checksum += a + b;
        }
    }
    EXPECT(rtopk_aggregate_workspace_bytes(1000, 0, 10, &bytes) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate_update_workspace_bytes(1000, 0, 10, &bytes) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate_update_workspace_bytes(1000, 2, 10, nullptr) == RTOPK_EINVAL);

    // ---- argument checks: nothing below is ever dereferenced or launched ----
    float *fake = reinterpret_cast<float *>(0x1000), *fake2 = reinterpret_cast<float *>(0x100000);
    uint32_t *fi = reinterpret_cast<uint32_t *>(0x2000);
    void *ws = reinterpret_cast<void *>(0x10000), *ws_odd = reinterpret_cast<void *>(0x10010);
    const uint64_t big = 1ull << 40;
    EXPECT(rtopk_encode(nullptr, fake2, 8, 4, 2, 0, 0, fi, fake, ws, big, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_encode(fake, fake2, 8, 4, 5, 0, 0, fi, fake, ws, big, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_encode(fake, fake, 8, 4, 2, 0, 0, fi, fake, ws, big, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_encode(fake, fake2, 8, 4, 2, 0, 0, fi, fake, ws, 16, nullptr) == RTOPK_EWORKSPACE);
    EXPECT(rtopk_encode(fake, fake2, 8, 4, 2, 0, 0, fi, fake, nullptr, big, nullptr) == RTOPK_EWORKSPACE);
    EXPECT(rtopk_encode(fake, fake2, 8, 4, 2, 0, 0, fi, fake, ws_odd, big, nullptr) == RTOPK_EWORKSPACE);
    {
        const float *g2[2] = {fake, reinterpret_cast<float *>(0x3000)};
        float *m2[2] = {fake2, reinterpret_cast<float *>(0x300000)};
        float *m_overlap[2] = {fake2, reinterpret_cast<float *>(0x3000)};
        uint32_t *oi[2] = {fi, fi + 64};
        float *ov[2] = {fake + 512, fake + 1024};
        const uint64_t seeds[2] = {1, 2};
        uint64_t one = 0;
        EXPECT(rtopk_encode_workspace_bytes(8, 4, 2, &one) == RTOPK_OK);
        EXPECT(rtopk_encode_batch(0, g2, m2, 8, 4, 2, seeds, 0, oi, ov, ws, big, nullptr) == RTOPK_EINVAL);
        EXPECT(rtopk_encode_batch(2, g2, m_overlap, 8, 4, 2, seeds, 0, oi, ov, ws, big, nullptr) == RTOPK_EINVAL);
        EXPECT(rtopk_encode_batch(2, g2, m2, 8, 4, 2, nullptr, 0, oi, ov, ws, big, nullptr) == RTOPK_EINVAL);
        EXPECT(rtopk_encode_batch(2, g2, m2, 8, 4, 2, seeds, 0, oi, ov, ws, one, nullptr) == RTOPK_EWORKSPACE);
        EXPECT(rtopk_encode_batch_device_step(2, g2, m2, 8, 4, 2, seeds, nullptr, oi, ov, ws, big,
                                              nullptr) == RTOPK_EINVAL);
        EXPECT(rtopk_encode_batch_device_step(2, g2, m2, 8, 4, 2, seeds,
                                              reinterpret_cast<const uint64_t *>(0x1004), oi, ov, ws,
                                              big, nullptr) == RTOPK_EINVAL);
    }
    EXPECT(rtopk_aggregate(nullptr, fake, 2, 3, 10, fake2, nullptr, 0, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate(fi, fake, 0, 3, 10, fake2, nullptr, 0, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate(fi, fake, 2, 3, 10, fake2, ws_odd, 0, nullptr) == RTOPK_EWORKSPACE);
    EXPECT(rtopk_aggregate_update(nullptr, fake, 2, 3, 10, 0.1f, 1.0f, fake2, ws, big, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate_update(fi, fake, 2, 3, 10, 0.1f, 1.0f, fake2, nullptr, big, nullptr) == RTOPK_EWORKSPACE);
    EXPECT(rtopk_aggregate_update(fi, fake, 2, 3, 10, 0.1f, 1.0f, fake2, ws, 8, nullptr) == RTOPK_EWORKSPACE);
    EXPECT(rtopk_aggregate_update(fi, fake, 70000, 3, 10, 0.1f, 1.0f, fake2, ws, big, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate_update_static(nullptr, fake, 2, 3, 10, 0.1f, 1.0f, fake2, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate_update_static(fi, fake, 32, 1, 1ull << 28, 0.1f, 1.0f, fake2, nullptr) == RTOPK_ETOOLARGE);
    EXPECT(rtopk_aggregate_update_momentum(fi, fake, 2, 3, 10, 0.1f, 1.0f, 0.9f, nullptr, fake2, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_aggregate_update_momentum(fi, fake, 2, 3, 10, 0.1f, 1.0f, 0.9f, fake2, fake2, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_diag_stream_add(fake, fake, 100, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_diag_stream_add(fake, reinterpret_cast<float *>(0x100004), 100, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_force_next_encode(64u) == RTOPK_EINVAL);
    EXPECT(rtopk_force_next_encode(RTOPK_FORCE_BRACKET_LOW | RTOPK_FORCE_BARRIER_TIMEOUT) == RTOPK_OK);
    EXPECT(rtopk_force_next_encode(RTOPK_FORCE_CHECK_IN_ABORT | RTOPK_FORCE_ESTIMATE_MISS) == RTOPK_OK);
    EXPECT(rtopk_force_next_encode(RTOPK_FORCE_KEY_WINDOW_MISS) == RTOPK_OK);
    EXPECT(rtopk_force_next_encode(0) == RTOPK_OK);
    EXPECT(rtopk_trace_next_encode(RTOPK_STAGE_FUSED, nullptr, nullptr) == RTOPK_EINVAL);
    EXPECT(rtopk_trace_next_encode(0, nullptr, nullptr) == RTOPK_OK);
    rtopk_encode_stats_t st;
    EXPECT(rtopk_encode_stats(nullptr, nullptr, &st) == RTOPK_EINVAL);
    for (int code = -6; code <= 0; ++code) EXPECT(std::strlen(rtopk_strerror(code)) > 0);
    EXPECT(rtopk_version() >= 200);
    std::printf("abi_driver: checksum %llu, %d failures\n", (unsigned long long)checksum, failures);
    return failures ? 1 : 0;
}
