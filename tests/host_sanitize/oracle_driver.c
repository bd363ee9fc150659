/*
 * Exercise of the CPU oracle for the sanitizer build: compiled together with
 * rtopk_oracle.c under AddressSanitizer and UndefinedBehaviorSanitizer, it
 * runs every oracle function over small inputs that reach the corners of the
 * index arithmetic (d = 1, k = r = d, ragged sizes, ties everywhere, repeated
 * and out-of-range indices, special values) and prints a checksum. It checks
 * memory safety and defined behaviour, not results: the pins do that.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void rtopk_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
uint64_t rtopk_oracle_key64(uint64_t seed, uint64_t step, uint32_t index);
int rtopk_oracle_top_r(const float *a, uint64_t d, uint64_t r, uint32_t *top_idx);
int rtopk_oracle_encode(const float *grad, float *residual, uint64_t d, uint64_t r, uint64_t k,
                        uint64_t seed, uint64_t step, uint32_t *out_idx, float *out_val);
int rtopk_oracle_aggregate(const uint32_t *idx, const float *val, uint32_t n, uint64_t k,
                           uint64_t d, float *out);
int rtopk_oracle_aggregate_f32(const uint32_t *idx, const float *val, uint32_t n, uint64_t k,
                               uint64_t d, float *out);
int rtopk_oracle_aggregate_update(const uint32_t *idx, const float *val, uint32_t n, uint64_t k,
                                  uint64_t d, double eta, double scale, const float *omega_in,
                                  float *omega_out);
int rtopk_oracle_aggregate_update_f32(const uint32_t *idx, const float *val, uint32_t n,
                                      uint64_t k, uint64_t d, float eta, float scale,
                                      const float *omega_in, float *omega_out);
int rtopk_oracle_aggregate_update_momentum(const uint32_t *idx, const float *val, uint32_t n,
                                           uint64_t k, uint64_t d, double eta, double scale,
                                           double mu, const float *omega_in, const float *vel_in,
                                           float *omega_out, float *vel_out);
int rtopk_oracle_aggregate_update_momentum_f32(const uint32_t *idx, const float *val, uint32_t n,
                                               uint64_t k, uint64_t d, float eta, float scale,
                                               float mu, const float *omega_in,
                                               const float *vel_in, float *omega_out,
                                               float *vel_out);

static uint64_t lcg = 88172645463325252ull;
static uint32_t next_u32(void)
{
    lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(lcg >> 32);
}

static uint64_t mix(uint64_t h, const void *p, size_t bytes)
{
    const unsigned char *c = (const unsigned char *)p;
    for (size_t i = 0; i < bytes; ++i) h = (h ^ c[i]) * 1099511628211ull;
    return h;
}

int main(void)
{
    uint64_t h = 1469598103934665603ull;
    int failures = 0;
    const uint64_t sizes[] = {1, 2, 3, 7, 64, 257, 1000, 4099};
    for (size_t si = 0; si < sizeof sizes / sizeof sizes[0]; ++si) {
        const uint64_t d = sizes[si];
        float *g = malloc(d * sizeof *g), *m = malloc(d * sizeof *m), *w = malloc(d * sizeof *w);
        float *v = malloc(d * sizeof *v), *o1 = malloc(d * sizeof *o1), *o2 = malloc(d * sizeof *o2);
        if (!g || !m || !w || !v || !o1 || !o2) return 2;
        for (int pattern = 0; pattern < 4; ++pattern) {
            for (uint64_t i = 0; i < d; ++i) {
                const uint32_t x = next_u32();
                float f;
                if (pattern == 0) f = (float)(int32_t)x * 1e-9f;          /* distinct values */
                else if (pattern == 1) f = (float)((int)(x % 3) - 1);      /* ties everywhere */
                else if (pattern == 2) f = 0.0f;                           /* all equal */
                else memcpy(&f, &x, sizeof f);                             /* any bit pattern */
                g[i] = f;
                m[i] = pattern == 3 ? 0.0f : (float)(x % 5) * 0.25f;
                w[i] = (float)(x % 11) - 5.0f;
                v[i] = (float)(x % 7) * 0.125f;
            }
            const uint64_t rs[] = {1, d / 3 + 1, d};
            for (int ri = 0; ri < 3; ++ri) {
                const uint64_t r = rs[ri] > d ? d : rs[ri];
                const uint64_t ks[] = {1, r / 2 + 1, r};
                for (int ki = 0; ki < 3; ++ki) {
                    const uint64_t k = ks[ki] > r ? r : ks[ki];
                    uint32_t *top = malloc(r * sizeof *top);
                    uint32_t *oi = malloc(2 * k * sizeof *oi);
                    float *ov = malloc(2 * k * sizeof *ov);
                    float *res = malloc(d * sizeof *res);
                    if (!top || !oi || !ov || !res) return 2;
                    memcpy(res, m, d * sizeof *res);
                    if (rtopk_oracle_top_r(g, d, r, top) != 0) ++failures;
                    h = mix(h, top, r * sizeof *top);
                    /* two workers: the second message behind the first */
                    if (rtopk_oracle_encode(g, res, d, r, k, 42, si, oi, ov) != 0) ++failures;
                    if (rtopk_oracle_encode(g, res, d, r, k, ~0ull, ~0ull - si, oi + k, ov + k) != 0)
                        ++failures;
                    h = mix(h, oi, 2 * k * sizeof *oi);
                    h = mix(h, res, d * sizeof *res);
                    if (rtopk_oracle_aggregate(oi, ov, 2, k, d, o1) != 0) ++failures;
                    h = mix(h, o1, d * sizeof *o1);
                    if (rtopk_oracle_aggregate_f32(oi, ov, 2, k, d, o1) != 0) ++failures;
                    h = mix(h, o1, d * sizeof *o1);
                    /* one worker with 2k entries: every index appears twice */
                    if (rtopk_oracle_aggregate_f32(oi, ov, 1, 2 * k, d, o1) != 0) ++failures;
                    if (rtopk_oracle_aggregate_update(oi, ov, 2, k, d, 0.1, 2.0, w, o1) != 0) ++failures;
                    if (rtopk_oracle_aggregate_update_f32(oi, ov, 2, k, d, 0.1f, 2.0f, w, o1) != 0)
                        ++failures;
                    h = mix(h, o1, d * sizeof *o1);
                    if (rtopk_oracle_aggregate_update_momentum(oi, ov, 2, k, d, 0.1, 2.0, 0.9, w, v,
                                                               o1, o2) != 0) ++failures;
                    if (rtopk_oracle_aggregate_update_momentum_f32(oi, ov, 2, k, d, 0.1f, 2.0f, 0.9f,
                                                                   w, v, o1, o2) != 0) ++failures;
                    h = mix(h, o2, d * sizeof *o2);
                    /* an index past the end must be refused, not written */
                    oi[2 * k - 1] = (uint32_t)d;
                    if (rtopk_oracle_aggregate(oi, ov, 2, k, d, o1) == 0) ++failures;
                    if (rtopk_oracle_aggregate_f32(oi, ov, 2, k, d, o1) == 0) ++failures;
                    if (rtopk_oracle_aggregate_update(oi, ov, 2, k, d, 0.1, 2.0, w, o1) == 0) ++failures;
                    free(top); free(oi); free(ov); free(res);
                }
            }
        }
        free(g); free(m); free(w); free(v); free(o1); free(o2);
    }
    /* the domain of Definition 3 */
    {
        float one = 1.0f, res = 0.0f, ov;
        uint32_t oi;
        if (rtopk_oracle_encode(&one, &res, 1, 1, 0, 0, 0, &oi, &ov) == 0) ++failures;
        if (rtopk_oracle_encode(&one, &res, 1, 2, 1, 0, 0, &oi, &ov) == 0) ++failures;
        if (rtopk_oracle_encode(&one, &res, 1, 1, 1, 0, 0, &oi, &ov) != 0) ++failures;
    }
    uint32_t ctr[4] = {~0u, ~0u, ~0u, ~0u}, key[2] = {~0u, ~0u}, out[4];
    rtopk_oracle_philox4x32_10(ctr, key, out);
    h = mix(h, out, sizeof out);
    h ^= rtopk_oracle_key64(~0ull, ~0ull, ~0u);
    printf("oracle_driver: checksum %016llx, %d failures\n", (unsigned long long)h, failures);
    return failures ? 1 : 0;
}
