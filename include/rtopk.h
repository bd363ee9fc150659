/*
 * rtopk.h -- C ABI of the MI355X (gfx950) rTop-k hot path.
 *
 * Two operations, both taken from the paper's problem statement (Section III,
 * Algorithm 1): per worker, sparsify the error-compensated gradient with the
 * rTop-k operator of Definition 3; on the master, average the n sparse
 * messages into one dense update.
 *
 * Conventions for every entry point
 *   - Pointers marked "device" are HIP device pointers valid on the current
 *     device; pointers marked "host" are ordinary host pointers.
 *   - The library allocates no device memory and never synchronises the host
 *     (rtopk_encode_stats excepted). All state that links one call to the
 *     next is in the caller's buffers (the residual) and arguments (step); the
 *     library itself only remembers, per device, the launch width of its
 *     streaming kernel. Work is enqueued on `stream` (a hipStream_t, may be
 *     NULL for the default stream) and the call returns at once. The caller
 *     owns all buffers, workspace included, and must keep them alive until the
 *     stream has drained.
 *   - The hot-path calls only launch kernels (what must start at zero is
 *     cleared by those kernels, not by memset nodes): they may be issued on a
 *     stream that is being captured into a HIP graph and replayed. A replay
 *     repeats the arguments it was captured with, the step number included:
 *     rtopk_encode and rtopk_encode_batch in a graph draw the SAME random
 *     subset on every replay, which under error feedback starves the members
 *     with large keys. A loop that replays a graph uses
 *     rtopk_encode_batch_device_step, which reads the step number from device
 *     memory that the graph itself advances.
 *   - Diagnostics (statistics of the last encode, event tracing, hooks that
 *     force the exact fallback paths, a streaming calibration kernel) are not
 *     part of this interface: they are declared in rtopk_diag.h.
 *   - Two calls may run concurrently only with distinct workspaces, residuals
 *     and outputs.
 *   - Return value: RTOPK_OK or a negative error code; rtopk_strerror() gives
 *     a static description. Argument checks are made on the host before
 *     anything is launched; a failed check launches nothing.
 *   - Results are a pure function of the argument values and buffer contents:
 *     they do not depend on grid size, stream or run, nor on what the
 *     workspace held. Against another
 *     implementation of the same arithmetic they agree bit for bit, with one
 *     exception IEEE 754 leaves open: when an addition meets two not-a-number
 *     operands with different payloads (two workers sending NaN for one
 *     coordinate; a NaN gradient entry on a NaN residual entry), the result is
 *     a NaN whose payload is the hardware's choice.
 */
#ifndef RTOPK_H
#define RTOPK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RTOPK_OK 0
#define RTOPK_EINVAL (-1)     /* null pointer, or sizes outside 1 <= k <= r <= d < 2^32, n < 1, aliasing */
#define RTOPK_EWORKSPACE (-2) /* workspace null, misaligned (256 bytes) or too small */
#define RTOPK_EHIP (-3)       /* a HIP call or kernel launch failed */
#define RTOPK_ETOOLARGE (-4)  /* sizes beyond the built-in scratch of rtopk_aggregate_update_static */

/* Bytes of device workspace one rtopk_encode call needs for these sizes: the
 * caller-owned scratch memory behind Algorithm 1's node-side step (nothing of
 * it survives the call). bytes: host pointer, written on success. */
int rtopk_encode_workspace_bytes(uint64_t d, uint64_t r, uint64_t k, uint64_t *bytes);

/* Bytes of device workspace rtopk_aggregate (Algorithm 1's master step) needs
 * for these sizes; currently 0, the argument is kept for the interface. */
int rtopk_aggregate_workspace_bytes(uint64_t d, uint32_t n, uint64_t k, uint64_t *bytes);

/*
 * One node-side step of Algorithm 1 for one worker:
 *     a <- grad + residual            (error compensation, one binary32 add)
 *     U <- rTop-k selection on a      (Definition 3: a uniformly random
 *                                      k-subset of the r largest-magnitude
 *                                      coordinates, Definition 1)
 *     message <- {(i, a_i) : i in U}
 *     residual <- a - message         (a_i where not sent; a_i - a_i where sent)
 *
 * Choices the paper leaves open, fixed here so the result is unique:
 *   magnitude order = order of the low 31 bits of the binary32 pattern; equal
 *   magnitudes: lower index first; U = the k members of the top-r set with
 *   the smallest (K(i), i), K(i) = first two output words (word0 << 32 |
 *   word1) of Philox4x32-10 with counter (i, 0, step_lo, step_hi) and key
 *   (seed_lo, seed_hi).
 *
 * grad       device, [d] binary32, read only
 * residual   device, [d] binary32, in: m_t, out: m_{t+1}; must not overlap grad
 * d, r, k    1 <= k <= r <= d < 2^32. r == k is the top-k operator (no key is
 *            ever computed), r == d the random-k operator (no magnitude is
 *            ever compared: no estimate, no histogram, no threshold)
 * seed,step  select the random subset; a fresh `step` gives a fresh subset,
 *            distinct `seed`s give independent workers
 * out_idx    device, [k] uint32, the set U in strictly ascending order
 * out_val    device, [k] binary32, out_val[j] = a[out_idx[j]]
 * workspace  device, 256-byte aligned, >= rtopk_encode_workspace_bytes(d,r,k):
 *            one byte per element (every chunk of the vector owns room for an
 *            eighth of its elements as 8-byte candidates; a chunk that keeps
 *            more is read from the residual buffer itself) plus about 10 MB
 *            of histograms, lists and counters; contents on entry are
 *            irrelevant, contents on return unspecified but for its first
 *            32-bit word: once the call's kernels have run it holds the
 *            call's error flags, 0 when the message is valid, non-zero when
 *            an internal consistency check failed (a selection found no
 *            element of its rank, the winners did not add up to k, a bounded
 *            wait inside a kernel ran out) and the outputs must be discarded.
 *            A caller that wants to know without stopping the stream copies
 *            that word asynchronously; no input in the domain above is known
 *            to set it
 * stream     hipStream_t
 */
int rtopk_encode(const float *grad, float *residual,
                 uint64_t d, uint64_t r, uint64_t k,
                 uint64_t seed, uint64_t step,
                 uint32_t *out_idx, float *out_val,
                 void *workspace, uint64_t workspace_bytes, void *stream);

/*
 * The same step of Algorithm 1 for n independent vectors of equal sizes in
 * one call: the n workers that Algorithm 1's node loop runs over (when one
 * device holds several of them), or the tensors of one model. Member i is
 * computed exactly as rtopk_encode(grad[i], residual[i], d, r, k, seed[i],
 * step, out_idx[i], out_val[i], ...) computes it, bit for bit; the members
 * only share kernel launches (up to 16 per launch), so the short kernels of
 * all members run side by side and the streaming kernel does not drain in
 * between.
 *
 * grad, residual, out_idx, out_val   HOST arrays of n device pointers each,
 *            read during the call; every pointer as for rtopk_encode. No two
 *            members may share or overlap a residual or an output buffer.
 * seed       HOST array of n seeds
 * workspace  device, 256-byte aligned, >= n * rtopk_encode_workspace_bytes(d,r,k);
 *            member i uses the i-th slice of that size (its first word holds
 *            member i's error flags), and rtopk_encode_stats on the slice's
 *            address reports on member i
 */
int rtopk_encode_batch(uint32_t n,
                       const float *const *grad, float *const *residual,
                       uint64_t d, uint64_t r, uint64_t k,
                       const uint64_t *seed, uint64_t step,
                       uint32_t *const *out_idx, float *const *out_val,
                       void *workspace, uint64_t workspace_bytes, void *stream);

/*
 * rtopk_encode_batch with the step number of Algorithm 1's loop read from
 * device memory when the kernels run, not passed by value when they are
 * enqueued: for a step captured once into a HIP graph and replayed every
 * iteration, with a small kernel in the same graph (or any other work on the
 * stream) advancing *step_device in between. Every replay then draws a fresh
 * uniform subset (Definition 3), as a loop of rtopk_encode_batch calls with
 * step = 0, 1, 2, ... does; the results are the same bit for bit.
 *
 * step_device   device, one uint64, 8-byte aligned; read by every kernel of
 *               the call, so it must not change while the call's kernels run
 * everything else as for rtopk_encode_batch (n = 1 serves a single vector)
 */
int rtopk_encode_batch_device_step(uint32_t n,
                                   const float *const *grad, float *const *residual,
                                   uint64_t d, uint64_t r, uint64_t k,
                                   const uint64_t *seed, const uint64_t *step_device,
                                   uint32_t *const *out_idx, float *const *out_val,
                                   void *workspace, uint64_t workspace_bytes, void *stream);

/*
 * Master step of Algorithm 1: out = (1/n) * sum_{w<n} message_w as a dense
 * vector. Every coordinate is divided by n, whether or not all workers sent
 * it; coordinates nobody sent are +0. Sums are formed in binary32 starting
 * from +0, adding workers in the order 0..n-1 (entries of one message in
 * position order, so a repeated index is simply added again), followed by
 * one correctly rounded binary32 division by (float)n. No floating-point
 * atomics are used, so the result is reproducible bit for bit.
 *
 * idx   device, [n*k] uint32, worker-major: worker w owns [w*k, (w+1)*k);
 *       each worker's slice must be sorted ascending (as rtopk_encode emits
 *       it); every index must be < d (precondition, not checked)
 * val   device, [n*k] binary32
 * out   device, [d] binary32, fully overwritten
 * workspace  device, 256-byte aligned, >= rtopk_aggregate_workspace_bytes
 */
int rtopk_aggregate(const uint32_t *idx, const float *val,
                    uint32_t n, uint64_t k, uint64_t d,
                    float *out,
                    void *workspace, uint64_t workspace_bytes, void *stream);

/*
 * Both master lines of Algorithm 1 in one step, without the dense average in
 * between: omega[i] <- omega[i] - eta * scale * (1/n) * sum_{w<n} message_w[i].
 * scale = 1 is the algorithm as printed. scale = r/k divides what a node kept
 * by the fraction k/r it kept of its top-r set, in the manner of the
 * estimator in the proof of the estimation upper bound, which divides the
 * subsampled vector by its subsampling fraction; the mean over the random
 * subsets then equals the top-r part of the node's vector.
 *
 * Arithmetic, all binary32: the sum and the division by n exactly as in
 * rtopk_aggregate; the step c = eta * scale rounded once; then one fused
 * multiply-add, omega[i] = fma(-c, average[i], omega[i]). A coordinate whose
 * average is zero (nobody sent it, what was sent cancels, or the quotient by
 * n underflows) is not written and keeps its bits; for finite c and omega[i]
 * that is the number the formula gives, up to the sign of a zero weight.
 * Reproducible bit for bit; no atomics.
 *
 * idx, val, n, k, d   as for rtopk_aggregate; n <= 65535
 * omega   device, [d] binary32, updated in place. Only weights that move are
 *         written; where many indices fall close together, the 16-byte groups
 *         around them are read and written back whole, the unmoved weights
 *         with the bits they had. Must not overlap idx, val or workspace.
 * workspace  device, 256-byte aligned, >= rtopk_aggregate_update_workspace_bytes
 *            (4 bytes per worker and per 2048 coordinates); contents on entry
 *            are irrelevant, contents on return unspecified
 * Errors: RTOPK_EINVAL, RTOPK_EWORKSPACE, RTOPK_EHIP as for rtopk_encode.
 */
int rtopk_aggregate_update_workspace_bytes(uint64_t d, uint32_t n, uint64_t k, uint64_t *bytes);
int rtopk_aggregate_update(const uint32_t *idx, const float *val,
                           uint32_t n, uint64_t k, uint64_t d,
                           float eta, float scale,
                           float *omega,
                           void *workspace, uint64_t workspace_bytes, void *stream);

/*
 * rtopk_aggregate_update for callers that cannot allocate device memory and
 * have no workspace to pass: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc. Same arguments, same kernels and
 * the same results bit for bit as rtopk_aggregate_update, but the table of
 * tile starts lives in a device array of RTOPK_STATIC_SCRATCH_BYTES that is
 * part of the library (every GPU the library runs on holds it until the
 * process ends). The call allocates nothing and calls no allocating routine.
 *
 * Limit: (ceil(d / 2048) + 1) * n * 4 bytes, rounded up to 256, must not
 * exceed RTOPK_STATIC_SCRATCH_BYTES (16 MiB: d = 2^28 with up to 31 workers,
 * d = 2^32 - 1 with one); beyond it the call returns RTOPK_ETOOLARGE and
 * launches nothing.
 * The first call on a device looks up the array's address (it may load the
 * library's device code): make it once outside any stream capture.
 * All calls on one GPU share the one array: two calls whose kernels may
 * overlap (different streams, no ordering between them) race; calls on one
 * stream, or ordered by events, are safe. Nothing in the array has to be
 * cleared between calls: every word a call reads it has written itself.
 */
#define RTOPK_STATIC_SCRATCH_BYTES (16u << 20)
int rtopk_aggregate_update_static(const uint32_t *idx, const float *val,
                                  uint32_t n, uint64_t k, uint64_t d,
                                  float eta, float scale,
                                  float *omega, void *stream);

/*
 * The master's update with momentum, the optimiser the experiments section
 * uses (momentum SGD; the paper prints no formula, this is the common one):
 *     ghat = (1/n) * sum_{w<n} message_w
 *     velocity[i] <- mu * velocity[i] + scale * ghat[i]
 *     omega[i]    <- omega[i] - eta * velocity[i]
 * for every i: the velocity decays where nothing was sent, so this is a dense
 * pass over both arrays (16 bytes per coordinate plus the messages). mu = 0
 * moves the weights as rtopk_aggregate_update does.
 *
 * Arithmetic, all binary32: the average exactly as in rtopk_aggregate;
 * u = scale * average (one rounding); velocity = fma(mu, velocity, u);
 * omega = fma(-eta, velocity, omega) with the rounded new velocity.
 * Reproducible bit for bit; no atomics, no workspace.
 *
 * idx, val, n, k, d   as for rtopk_aggregate
 * omega, velocity     device, [d] binary32 each, updated in place; they must
 *                     not overlap each other, idx or val
 */
int rtopk_aggregate_update_momentum(const uint32_t *idx, const float *val,
                                    uint32_t n, uint64_t k, uint64_t d,
                                    float eta, float scale, float mu,
                                    float *omega, float *velocity, void *stream);

const char *rtopk_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int rtopk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RTOPK_H */
