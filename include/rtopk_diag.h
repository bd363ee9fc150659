/*
 * rtopk_diag.h -- diagnostics of the rTop-k library: statistics of the last
 * encode, HIP-event tracing of its stages, hooks that force its exact fallback
 * paths, and a streaming calibration kernel. Tests, benchmarks and profiling
 * use these; a training loop needs none of them. The interface proper is
 * rtopk.h. Everything here is for eager use (not under stream capture).
 */
#ifndef RTOPK_DIAG_H
#define RTOPK_DIAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Diagnostics of the most recent rtopk_encode that used `workspace`.
 * Synchronises `stream`, then copies a few counters to the host. Not part of
 * the hot path; tests and profiling use it.
 */
typedef struct rtopk_encode_stats {
    uint32_t error_flags;        /* 0 = clean; bit 1: a selection found no element of the requested
                                    rank; bit 2: the winners did not add up to k; bit 3: a workgroup
                                    of the many-workgroup selection gave up waiting for the others
                                    (any bit set: results invalid) */
    uint32_t path;               /* 0: both cut points came from the short lists; bit 0: at least one
                                    came from the slow selection over all candidates; bit 1: the
                                    sampled estimate failed and the vector itself was walked;
                                    bit 2: the threshold lies in a run of equal magnitudes too long
                                    for the short list (zeros, signs, a few quantisation levels):
                                    its last member was located from per-chunk counts; bit 3: the
                                    selection over all candidates ran on many workgroups (vectors
                                    of 256 chunks or more) */
    uint32_t threshold_bits;     /* magnitude pattern of the r-th largest |a_i|. With r == d no
                                    magnitude is looked at: threshold_bits and count_greater
                                    are reported as 0 and ties_taken as r */
    uint32_t boundary_list_size; /* candidates that shared the deciding histogram bin */
    uint64_t count_greater;      /* #{i : mag(a_i) > threshold} */
    uint64_t ties_taken;         /* r - count_greater, taken from the lowest indices */
    uint64_t superset_size;      /* entries compacted before the exact selection */
    uint64_t key_list_size;      /* members whose sampling key fell inside the a-priori window */
} rtopk_encode_stats_t;

int rtopk_encode_stats(const void *workspace, void *stream, rtopk_encode_stats_t *host_out);

/*
 * Instrumentation for benchmarks: the NEXT rtopk_encode issued from the
 * calling host thread records `ev_begin` (a hipEvent_t) on its stream right
 * before the kernels of `stage` and `ev_end` right after them; the request is
 * then forgotten. Stage RTOPK_STAGE_ALL brackets the whole call. The events
 * stay owned by the caller. Passing stage 0 cancels a pending request.
 */
#define RTOPK_STAGE_PREPARE 1   /* sample a = g + m, estimate the threshold range, clear counters */
#define RTOPK_STAGE_FUSED 2     /* a = g + m, store, candidates + histogram */
#define RTOPK_STAGE_CLASSIFY 3  /* certain members, key window, short lists */
#define RTOPK_STAGE_FINALIZE 4  /* exact cut points, output offsets */
#define RTOPK_STAGE_EMIT 5      /* message + residual write-back */
#define RTOPK_STAGE_ALL 100
int rtopk_trace_next_encode(int stage, void *ev_begin, void *ev_end);

/*
 * Test hook: the NEXT rtopk_encode issued from the calling host thread behaves
 * as if one of its two statistical shortcuts had failed, so that the exact
 * fallbacks behind them can be exercised on ordinary inputs; the request is
 * then forgotten. The results must not change, only rtopk_encode_stats.path
 * (RTOPK_FORCE_BARRIER_TIMEOUT excepted, see there).
 *   RTOPK_FORCE_ESTIMATE_MISS    the sampled threshold estimate keeps no
 *                                candidates: the vector itself is walked
 *   RTOPK_FORCE_KEY_WINDOW_MISS  the a-priori window around the k-th smallest
 *                                sampling key is empty: the key cut comes from
 *                                a selection over all candidates
 *   RTOPK_FORCE_CHECK_IN_ABORT   when the exact selection over all candidates
 *                                is about to run on many workgroups, they
 *                                decide at check-in that they are not all
 *                                resident (as when another stream's grid holds
 *                                compute units and waits too): one workgroup
 *                                runs the selection alone. Only has an effect
 *                                together with a condition that needs the
 *                                selection.
 *   RTOPK_FORCE_BRACKET_LOW      the estimate's upper bound is put at its lower
 *                                bound, as if the sample had underestimated
 *                                the r-th largest magnitude: the threshold
 *                                then lies above the finely binned range, in
 *                                the one bin that holds everything above it
 *   RTOPK_FORCE_BARRIER_TIMEOUT  (an error path, not a fallback) the bounded
 *                                waits between the workgroups of the
 *                                many-workgroup selection give up at their
 *                                first poll: every kernel still ends normally,
 *                                error_flags reports bit 3, and the outputs of
 *                                that call are invalid. Only has an effect
 *                                together with a condition that needs the
 *                                selection on a vector of 256 chunks or more.
 * Passing 0 cancels a pending request.
 */
#define RTOPK_FORCE_ESTIMATE_MISS 1u
#define RTOPK_FORCE_KEY_WINDOW_MISS 2u
#define RTOPK_FORCE_CHECK_IN_ABORT 4u
#define RTOPK_FORCE_BRACKET_LOW 8u
#define RTOPK_FORCE_BARRIER_TIMEOUT 16u
int rtopk_force_next_encode(unsigned flags);

/*
 * Calibration: residual[i] <- grad[i] + residual[i] for i < d and nothing
 * else, streamed exactly as the encoder's dominant kernel streams its three
 * arrays (same grid, same 16-byte accesses with the streaming hint, same
 * chunking), so that what a read-read-write stream of 12 d bytes reaches on
 * this memory system can be measured beside that kernel.
 * grad, residual: device, 16-byte aligned, d elements, not overlapping.
 */
int rtopk_diag_stream_add(const float *grad, float *residual, uint64_t d, void *stream);

/*
 * 1 when the library was built with RTOPK_DEBUG_CHECKS, else 0. In that build
 * rtopk_aggregate, rtopk_aggregate_update, rtopk_aggregate_update_static and
 * rtopk_aggregate_update_momentum first verify on the device that every index
 * is below d and every worker's slice ascends, synchronise the stream and
 * return RTOPK_EINVAL if not; in the release build these stay preconditions.
 */
int rtopk_debug_checks(void);

#ifdef __cplusplus
}
#endif
#endif /* RTOPK_DIAG_H */
