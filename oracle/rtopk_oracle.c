/*
 * CPU oracle for the rTop-k sparsifier with error compensation and for the
 * master's averaging step.
 *
 * THIS FILE IS TEST INFRASTRUCTURE. It is the slow, plain statement of what
 * the HIP library must compute, written from the paper's definitions. Only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may call
 * it; the product path never does, and the two share no code.
 *
 * What is computed, and where the paper defines it:
 *   - top_r          Definition 1 (top-r sparsification): keep the r entries
 *                    that come first under a permutation ordering the entries
 *                    by non-increasing magnitude.
 *   - encode         Definition 3 (rTop-k) inside Algorithm 1's node loop:
 *                    g <- g + m ; ghat <- rTop_k(g) ; m <- g - ghat.
 *   - aggregate      Algorithm 1, master: ghat <- (1/n) sum_i ghat_i.
 *   - aggregate_update  the master's two lines together:
 *                    omega <- omega - eta * scale * (1/n) sum_i ghat_i.
 *                    scale = 1 is Algorithm 1 as printed; scale = r/k divides
 *                    what a node kept by the fraction k/r it kept of its
 *                    top-r set, the way the estimator in the proof of the
 *                    estimation upper bound divides the subsampled vector by
 *                    its subsampling fraction (unbiased for the top-r part).
 *
 * Readings taken where the paper leaves a choice open (they make the result
 * unique, so that another implementation can be compared bit for bit):
 *   - Magnitude order is the order of the 31 low bits of the binary32 pattern
 *     (identical to |x| order for finite values; +0 and -0 tie).
 *   - Among equal magnitudes the lower index comes first in the permutation.
 *   - The k-subset U of the top-r set, which Definition 3 draws uniformly
 *     among all k-subsets: every member i of the top-r set gets the 64-bit key
 *         K(i) = Philox4x32-10(counter = (i, 0, step_lo, step_hi),
 *                              key     = (seed_lo, seed_hi)),
 *         K = (out0 << 32) | out1,
 *     and U is the k members with the smallest (K, i). Ranking i.i.d. keys
 *     yields a uniformly distributed k-subset. Philox4x32-10 is the public
 *     counter-based generator of Salmon, Moraes, Dror and Shaw (SC'11).
 *   - Arithmetic is IEEE binary32: one rounded add for g + m, one rounded
 *     subtract for g - ghat. The message lists (index, value) pairs in
 *     ascending index order.
 *   - The master divides by n, the number of workers, for every coordinate
 *     (Algorithm 1), not by the number of workers that sent it.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)
#define ORACLE_ENOMEM (-2)

/* ------------------------------------------------------------------------
 * Philox4x32-10 (Salmon et al., SC'11).
 * State: counter c[0..3], key k[0..1]. One round:
 *   (hi0, lo0) = 0xD2511F53 * c0      (32x32 -> 64 bit product)
 *   (hi1, lo1) = 0xCD9E8D57 * c2
 *   c <- (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0)
 * Ten rounds; between rounds the key is bumped by the Weyl constants
 * (0x9E3779B9, 0xBB67AE85) modulo 2^32.
 * ---------------------------------------------------------------------- */
void rtopk_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                                uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 64-bit sampling key of coordinate `index` at (seed, step). */
uint64_t rtopk_oracle_key64(uint64_t seed, uint64_t step, uint32_t index)
{
    uint32_t ctr[4] = { index, 0u, (uint32_t)step, (uint32_t)(step >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    rtopk_oracle_philox4x32_10(ctr, key, out);
    return ((uint64_t)out[0] << 32) | (uint64_t)out[1];
}

/* ------------------------------------------------------------------------ */
static uint32_t magnitude_bits(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    return u & 0x7FFFFFFFu;
}

typedef struct { uint32_t mag; uint32_t idx; } mag_idx_t;
typedef struct { uint64_t key; uint32_t idx; } key_idx_t;

/* larger magnitude first; equal magnitudes: lower index first */
static int by_mag_desc_idx_asc(const void *pa, const void *pb)
{
    const mag_idx_t *a = (const mag_idx_t *)pa, *b = (const mag_idx_t *)pb;
    if (a->mag != b->mag) return a->mag > b->mag ? -1 : 1;
    if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
    return 0;
}

/* smaller key first; equal keys: lower index first */
static int by_key_asc_idx_asc(const void *pa, const void *pb)
{
    const key_idx_t *a = (const key_idx_t *)pa, *b = (const key_idx_t *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->idx != b->idx) return a->idx < b->idx ? -1 : 1;
    return 0;
}

static int by_u32_asc(const void *pa, const void *pb)
{
    uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

static int check_domain(uint64_t d, uint64_t r, uint64_t k)
{
    /* Definition 3: 1 <= k <= r <= d; indices are 32-bit */
    if (k < 1 || k > r || r > d || d > 0xFFFFFFFFull) return ORACLE_EINVAL;
    return ORACLE_OK;
}

/*
 * Definition 1. Writes pi(1..r), i.e. the indices of the r entries of `a`
 * that come first when all d entries are fully sorted by (magnitude
 * descending, index ascending), in that order.
 */
int rtopk_oracle_top_r(const float *a, uint64_t d, uint64_t r, uint32_t *top_idx)
{
    if (!a || !top_idx || r < 1 || r > d || d > 0xFFFFFFFFull) return ORACLE_EINVAL;
    mag_idx_t *all = (mag_idx_t *)malloc((size_t)d * sizeof *all);
    if (!all) return ORACLE_ENOMEM;
    for (uint64_t i = 0; i < d; ++i) {
        all[i].mag = magnitude_bits(a[i]);
        all[i].idx = (uint32_t)i;
    }
    qsort(all, (size_t)d, sizeof *all, by_mag_desc_idx_asc);
    for (uint64_t j = 0; j < r; ++j) top_idx[j] = all[j].idx;
    free(all);
    return ORACLE_OK;
}

/*
 * One node-side step of Algorithm 1 for one worker.
 *   grad      [d] in    g_i^t
 *   residual  [d] inout m_i^t on entry, m_i^{t+1} on return
 *   out_idx   [k] out   the set U in ascending order
 *   out_val   [k] out   (g + m) at those indices
 */
int rtopk_oracle_encode(const float *grad, float *residual,
                        uint64_t d, uint64_t r, uint64_t k,
                        uint64_t seed, uint64_t step,
                        uint32_t *out_idx, float *out_val)
{
    if (!grad || !residual || !out_idx || !out_val) return ORACLE_EINVAL;
    int rc = check_domain(d, r, k);
    if (rc) return rc;

    float *acc = (float *)malloc((size_t)d * sizeof *acc);
    float *ghat = (float *)calloc((size_t)d, sizeof *ghat);
    uint32_t *top = (uint32_t *)malloc((size_t)r * sizeof *top);
    key_idx_t *keyed = (key_idx_t *)malloc((size_t)r * sizeof *keyed);
    if (!acc || !ghat || !top || !keyed) {
        free(acc); free(ghat); free(top); free(keyed);
        return ORACLE_ENOMEM;
    }

    /* error compensation (Algorithm 1, node loop): the memory is added to the
       fresh gradient, one rounded binary32 addition per coordinate */
    for (uint64_t i = 0; i < d; ++i) {
        volatile float s = grad[i] + residual[i];
        acc[i] = s;
    }

    /* Definition 1: the top-r set, by a full sort */
    rc = rtopk_oracle_top_r(acc, d, r, top);
    if (rc) { free(acc); free(ghat); free(top); free(keyed); return rc; }

    /* Definition 3: k of those r, the ones whose (key, index) is smallest;
       the message lists them by ascending index */
    for (uint64_t j = 0; j < r; ++j) {
        keyed[j].idx = top[j];
        keyed[j].key = rtopk_oracle_key64(seed, step, top[j]);
    }
    qsort(keyed, (size_t)r, sizeof *keyed, by_key_asc_idx_asc);
    for (uint64_t j = 0; j < k; ++j) out_idx[j] = keyed[j].idx;
    qsort(out_idx, (size_t)k, sizeof *out_idx, by_u32_asc);

    /* the sparsified vector: a on U, zero elsewhere */
    for (uint64_t j = 0; j < k; ++j) {
        ghat[out_idx[j]] = acc[out_idx[j]];
        out_val[j] = acc[out_idx[j]];
    }

    /* the new memory is what was not sent: one rounded binary32 subtraction
       per coordinate */
    for (uint64_t i = 0; i < d; ++i) {
        volatile float e = acc[i] - ghat[i];
        residual[i] = e;
    }

    free(acc); free(ghat); free(top); free(keyed);
    return ORACLE_OK;
}

/*
 * Master step of Algorithm 1: out = (1/n) * sum over workers of their sparse
 * vectors. idx/val are worker-major: worker w owns entries [w*k, (w+1)*k).
 * The sum is accumulated in binary64 in worker order, divided by n in
 * binary64 and rounded once to binary32. An index that appears more than
 * once inside one message is summed like any other entry.
 */
int rtopk_oracle_aggregate(const uint32_t *idx, const float *val,
                           uint32_t n, uint64_t k, uint64_t d, float *out)
{
    if (!idx || !val || !out || n < 1 || k < 1 || d < 1 || d > 0xFFFFFFFFull)
        return ORACLE_EINVAL;
    double *acc = (double *)calloc((size_t)d, sizeof *acc);
    if (!acc) return ORACLE_ENOMEM;
    for (uint32_t w = 0; w < n; ++w)
        for (uint64_t j = 0; j < k; ++j) {
            uint32_t i = idx[(uint64_t)w * k + j];
            if (i >= d) { free(acc); return ORACLE_EINVAL; }
            acc[i] += (double)val[(uint64_t)w * k + j];
        }
    for (uint64_t i = 0; i < d; ++i) out[i] = (float)(acc[i] / (double)n);
    free(acc);
    return ORACLE_OK;
}

/*
 * The same average carried out entirely in binary32: partial sums start at
 * +0, workers are added in the order 0..n-1 (entries of one worker in
 * position order), then one binary32 division by (float)n. This is what an
 * fp32 implementation that adds in worker order produces bit for bit.
 */
int rtopk_oracle_aggregate_f32(const uint32_t *idx, const float *val,
                               uint32_t n, uint64_t k, uint64_t d, float *out)
{
    if (!idx || !val || !out || n < 1 || k < 1 || d < 1 || d > 0xFFFFFFFFull)
        return ORACLE_EINVAL;
    for (uint64_t i = 0; i < d; ++i) out[i] = 0.0f;
    for (uint32_t w = 0; w < n; ++w)
        for (uint64_t j = 0; j < k; ++j) {
            uint32_t i = idx[(uint64_t)w * k + j];
            if (i >= d) return ORACLE_EINVAL;
            volatile float s = out[i] + val[(uint64_t)w * k + j];
            out[i] = s;
        }
    const float fn = (float)n;
    for (uint64_t i = 0; i < d; ++i) {
        volatile float q = out[i] / fn;
        out[i] = q;
    }
    return ORACLE_OK;
}

/*
 * Master step of Algorithm 1 with the weight update folded in:
 *     omega_out = omega_in - eta * scale * (1/n) * sum_i ghat_i
 * for EVERY coordinate, exactly as the algorithm's master lines read: a
 * coordinate nobody sent has ghat = 0 and goes through the same subtraction.
 * Sum in binary64 in worker order, everything else in binary64, one rounding
 * to binary32 at the end. omega_in and omega_out may be the same array.
 */
int rtopk_oracle_aggregate_update(const uint32_t *idx, const float *val,
                                  uint32_t n, uint64_t k, uint64_t d,
                                  double eta, double scale,
                                  const float *omega_in, float *omega_out)
{
    if (!idx || !val || !omega_in || !omega_out || n < 1 || k < 1 || d < 1 ||
        d > 0xFFFFFFFFull)
        return ORACLE_EINVAL;
    double *acc = (double *)calloc((size_t)d, sizeof *acc);
    if (!acc) return ORACLE_ENOMEM;
    for (uint32_t w = 0; w < n; ++w)
        for (uint64_t j = 0; j < k; ++j) {
            uint32_t i = idx[(uint64_t)w * k + j];
            if (i >= d) { free(acc); return ORACLE_EINVAL; }
            acc[i] += (double)val[(uint64_t)w * k + j];
        }
    for (uint64_t i = 0; i < d; ++i) {
        const double ghat = acc[i] / (double)n;
        omega_out[i] = (float)((double)omega_in[i] - eta * scale * ghat);
    }
    free(acc);
    return ORACLE_OK;
}

/*
 * The same update in binary32 with a fixed order of operations: the average
 * exactly as rtopk_oracle_aggregate_f32 forms it (sum from +0 in worker
 * order, one division by (float)n), the step c = (float)eta * (float)scale
 * rounded once, and omega_out = fma(-c, average, omega_in) with the single
 * rounding of a fused multiply-add. Reading taken for binary32 only (the
 * binary64 form above is the algorithm's line as it stands): a coordinate
 * whose AVERAGE is zero (nobody sent it, what was sent cancels, or the
 * quotient by n underflows) keeps its weight bit for bit, it is copied. For
 * finite c and w that is the number fma(-c, 0, w) gives, up to the sign of a
 * zero weight; a signalling not-a-number stays signalling.
 */
int rtopk_oracle_aggregate_update_f32(const uint32_t *idx, const float *val,
                                      uint32_t n, uint64_t k, uint64_t d,
                                      float eta, float scale,
                                      const float *omega_in, float *omega_out)
{
    if (!idx || !val || !omega_in || !omega_out || n < 1 || k < 1 || d < 1 ||
        d > 0xFFFFFFFFull)
        return ORACLE_EINVAL;
    float *avg = (float *)malloc((size_t)d * sizeof *avg);
    if (!avg) return ORACLE_ENOMEM;
    int rc = rtopk_oracle_aggregate_f32(idx, val, n, k, d, avg);
    if (rc != ORACLE_OK) { free(avg); return rc; }
    volatile float c = eta * scale;
    const float neg_c = -c;
    for (uint64_t i = 0; i < d; ++i)
        omega_out[i] = avg[i] != 0.0f ? fmaf(neg_c, avg[i], omega_in[i]) : omega_in[i];
    free(avg);
    return ORACLE_OK;
}

/*
 * The master's update with momentum, the optimiser the experiments section
 * names (momentum SGD; the paper gives no formula, this is the common one):
 *     ghat = (1/n) sum_i ghat_i
 *     v    <- mu * v + scale * ghat
 *     w    <- w - eta * v
 * for every coordinate (the velocity decays where nothing was sent). mu = 0
 * is Algorithm 1's plain step. binary64 throughout, one rounding per output.
 */
int rtopk_oracle_aggregate_update_momentum(const uint32_t *idx, const float *val,
                                           uint32_t n, uint64_t k, uint64_t d,
                                           double eta, double scale, double mu,
                                           const float *omega_in, const float *vel_in,
                                           float *omega_out, float *vel_out)
{
    if (!idx || !val || !omega_in || !vel_in || !omega_out || !vel_out || n < 1 || k < 1 ||
        d < 1 || d > 0xFFFFFFFFull)
        return ORACLE_EINVAL;
    double *acc = (double *)calloc((size_t)d, sizeof *acc);
    if (!acc) return ORACLE_ENOMEM;
    for (uint32_t w = 0; w < n; ++w)
        for (uint64_t j = 0; j < k; ++j) {
            uint32_t i = idx[(uint64_t)w * k + j];
            if (i >= d) { free(acc); return ORACLE_EINVAL; }
            acc[i] += (double)val[(uint64_t)w * k + j];
        }
    for (uint64_t i = 0; i < d; ++i) {
        const double ghat = acc[i] / (double)n;
        const double v = mu * (double)vel_in[i] + scale * ghat;
        vel_out[i] = (float)v;
        omega_out[i] = (float)((double)omega_in[i] - eta * v);
    }
    free(acc);
    return ORACLE_OK;
}

/*
 * The same in binary32 with a fixed order of operations: the average as
 * rtopk_oracle_aggregate_f32 forms it, u = scale * average (one rounding),
 * v' = fma(mu, v, u), w' = fma(-eta, v', w), where v' is the ROUNDED new
 * velocity (the one that is stored).
 */
int rtopk_oracle_aggregate_update_momentum_f32(const uint32_t *idx, const float *val,
                                               uint32_t n, uint64_t k, uint64_t d,
                                               float eta, float scale, float mu,
                                               const float *omega_in, const float *vel_in,
                                               float *omega_out, float *vel_out)
{
    if (!idx || !val || !omega_in || !vel_in || !omega_out || !vel_out || n < 1 || k < 1 ||
        d < 1 || d > 0xFFFFFFFFull)
        return ORACLE_EINVAL;
    float *avg = (float *)malloc((size_t)d * sizeof *avg);
    if (!avg) return ORACLE_ENOMEM;
    int rc = rtopk_oracle_aggregate_f32(idx, val, n, k, d, avg);
    if (rc != ORACLE_OK) { free(avg); return rc; }
    const float neg_eta = -eta;
    for (uint64_t i = 0; i < d; ++i) {
        volatile float u = scale * avg[i];
        const float v = fmaf(mu, vel_in[i], u);
        vel_out[i] = v;
        omega_out[i] = fmaf(neg_eta, v, omega_in[i]);
    }
    free(avg);
    return ORACLE_OK;
}
