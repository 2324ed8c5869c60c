/*
 * wash.h -- C ABI of the MI355X (gfx950) population-update library for WASH
 * ("Train your Ensemble with Communication-Efficient Weight Shuffling, then
 * Average", arXiv 2405.17517).
 *
 * The population of N models lives on ONE GPU as a stacked, row-major [N, P]
 * fp32 buffer (row n = all parameters of model n, tensors concatenated without
 * padding; row stride = P elements), optionally with a second [N, P] buffer of
 * optimizer state (SGD momentum).  Three operations act on it:
 *
 *   wash_shuffle   the shuffling step            (Sec. 3, Eq. 3; Alg. 1, shuffling step)
 *   wash_average   the final uniform average     (Alg. 1, output line)
 *   papa_ema       PAPA's EMA toward the mean    (Sec. 3, Eq. 1)  -- comparison baseline
 *
 * one host helper gives the layer-wise probabilities of Eq. 6, and two further
 * passes serve the paper's analysis: wash_consensus_sqdist (Eq. 2, Eq. 5) and
 * wash_weighted_average (interpolations between the models).  Measurement
 * aids (a plain copy, a scattered-access probe) are declared in wash_bench.h.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory on the CURRENT device of the
 *     calling thread; "host" pointers are ordinary process memory.
 *   - The caller owns every buffer it passes.  The library allocates only a
 *     small internal device table per distinct segment list (cached), and, per
 *     stream that asks for a selected count, a step advance or a consensus
 *     distance, one workspace of about 1 MiB (plus a few spare ones, for
 *     streams under graph capture, which cannot allocate), on first use;
 *     wash_shutdown() releases them.  Calls on different streams never share
 *     a workspace; wash_consensus_sqdist_noalloc is the one call that uses a
 *     fixed array instead.  At most 256 workspaces exist: when a process has
 *     used more streams than that, the call that needs another one waits for
 *     the device to become idle and takes back those of ordinary streams
 *     (workspaces recorded into graphs stay with their graphs).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without waiting; the usual stream
 *     ordering applies to the buffers.
 *   - Return value: WASH_OK (0) or a negative wash_status.  Arguments are
 *     validated before anything is launched: on WASH_EINVAL nothing was
 *     modified.  Nothing throws or aborts.  wash_strerror() gives the text,
 *     wash_last_error_detail() the detail of the calling thread's last error.
 */
#ifndef WASH_H
#define WASH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define WASH_MAX_N 32u /* largest population size accepted */
#define WASH_MAX_STATES 4 /* buffers wash_shuffle_states moves together: parameters + 3 optimizer states */

typedef enum wash_status {
    WASH_OK = 0,
    WASH_EINVAL = -1, /* an argument violates the contract below */
    WASH_EHIP = -2,   /* a HIP call (launch, copy, allocation) failed */
    WASH_ENOMEM = -3  /* host allocation failed */
} wash_status;

/*
 * One tensor ("layer" in the sense of Eq. 6 is the caller's business: the
 * library takes one probability per segment).  Coordinates are positions in a
 * row, 0 <= offset, offset + length <= P.
 */
typedef struct wash_segment {
    uint64_t offset; /* first coordinate of the segment */
    uint64_t length; /* number of coordinates (0 allowed) */
    double p;        /* probability that a coordinate of it is shuffled, in [0, 1] */
} wash_segment;

/*
 * The shuffling step, Eq. 3 / Alg. 1: for every coordinate g of every segment,
 * independently with probability p of its segment, draw a permutation pi_g
 * uniform on all N! permutations (independent of the Bernoulli draw) and set
 * params[n][g] <- params_old[pi_g(n)][g] for all n at once.  The draw is one
 * per coordinate, shared by the N models, so each coordinate's multiset of
 * values, the population mean and the consensus distance (Eq. 5) are kept.
 * If `momentum` is given, the same mask and the same pi_g move it too (the
 * WASH+Opt variant, Sec. 4).  Values are moved as raw 32-bit patterns.
 *
 * Randomness is a pure function of (seed, step, g, N, p): the same arguments
 * give the same bits whatever the launch shape, however a tensor is cut into
 * segments of equal p, and whether or not momentum is passed.  Stream "v1":
 * Philox4x32-10 keyed by seed; mask word of g = word (g mod 4) of the call at
 * counter (g/4, step, 0), selected iff word < round(p * 2^32); permutation
 * words from counters (g, step, 1 + t/4); descending Fisher-Yates with
 * multiply-high range reduction.
 *
 *   params          device, [N, P] fp32, updated in place
 *   momentum        device, [N, P] fp32 or NULL; must not overlap params
 *   N               population size, 1 .. WASH_MAX_N   (N = 1: identity)
 *   P               coordinates per model, >= 1
 *   segs            HOST array of nsegs segments, sorted by offset and not
 *                   overlapping; read before the call returns.  Coordinates in
 *                   no segment are never shuffled.  (Inside segments with
 *                   p >= 0.08 the rows are streamed through on-chip memory in
 *                   aligned strips of 256 coordinates, and the call may rewrite
 *                   any element of such a strip with the value it already has;
 *                   see WASH_OPT_DENSE.)
 *   nsegs           number of segments (0 allowed: nothing happens)
 *                   (A list seen for the first time costs one device allocation and
 *                   one blocking copy of a small table; the 16 most recent lists per
 *                   process are kept, and dropping an older one waits for the
 *                   device.  The paper's probabilities do not change over the
 *                   iterations; a caller that changes them every step pays this
 *                   every step.)
 *   seed, step      stream address; step < 2^32
 *   selected_count  device uint64 or NULL; the number of selected coordinates
 *                   (the per-model communication volume of Sec. 3) is ADDED to it
 *   stream          hipStream_t
 *
 * Errors: WASH_EINVAL for NULL params, N = 0 or > WASH_MAX_N, P = 0, a
 * probability outside [0, 1] or NaN, a segment outside [0, P), unsorted or
 * overlapping segments, step >= 2^32, momentum == params; WASH_EHIP if a HIP
 * call fails.
 */
int wash_shuffle(float *params, float *momentum, uint32_t N, uint64_t P,
                 const wash_segment *segs, uint32_t nsegs,
                 uint64_t seed, uint64_t step,
                 uint64_t *selected_count, void *stream);

/*
 * The same shuffling step (Eq. 3, same law, same arguments, same errors) on a
 * second random stream, "gap": instead of one Bernoulli draw per coordinate the
 * distances between successive selected coordinates are drawn (geometric, by
 * inversion: 1 + floor(log2(u) / log2(1-p)); the walk restarts at every
 * multiple of 1024 coordinates and at every segment start, which keeps the
 * trials independent because the geometric law has no memory).  The random-number
 * work is then proportional to the number of SELECTED coordinates, p * P per
 * step, the quantity the paper counts as communication volume (Sec. 3), instead
 * of P.  The permutation of a selected coordinate is the one of wash_shuffle.
 * A segment whose p is so small that 1 - p rounds to 1 in double (p <= 2^-54)
 * selects nothing, like p = 0: Bernoulli(p) to within 2^-54 per coordinate.
 * Results differ bit for bit from wash_shuffle (different mask), are the same
 * in law, and are a pure function of (seed, step, N, and the segment list after
 * dropping empty segments and merging touching neighbours of equal p).
 */
int wash_shuffle_gap(float *params, float *momentum, uint32_t N, uint64_t P,
                     const wash_segment *segs, uint32_t nsegs,
                     uint64_t seed, uint64_t step,
                     uint64_t *selected_count, void *stream);

/*
 * WASH+Opt (Sec. 4, the variant that also permutes the optimizer state of a
 * shuffled parameter) for optimizers with more than one state per parameter,
 * e.g. Adam's two moment estimates: every buffer is permuted with the same mask
 * and the same permutation per coordinate, in one pass.  wash_shuffle(params,
 * momentum, ...) is the case nbuffers = 1 or 2 with gap_stream = 0, and
 * wash_shuffle_gap the same with gap_stream = 1; the result on each buffer is
 * bit-identical to what those calls give for that buffer alone.
 *   buffers     HOST array of nbuffers device pointers, each [N, P] fp32 with row
 *               stride P; buffers[0] is the parameter population; no two may overlap;
 *               the array is read before the call returns
 *   nbuffers    1 .. WASH_MAX_STATES
 *   gap_stream  0: the stream of wash_shuffle; 1: the stream of wash_shuffle_gap
 *   others      as for wash_shuffle
 * Errors: as for wash_shuffle, plus WASH_EINVAL for buffers = NULL, a NULL entry,
 * nbuffers = 0 or > WASH_MAX_STATES, gap_stream not 0 or 1.
 */
int wash_shuffle_states(float *const *buffers, uint32_t nbuffers, uint32_t N, uint64_t P,
                        const wash_segment *segs, uint32_t nsegs,
                        uint64_t seed, uint64_t step, int gap_stream,
                        uint64_t *selected_count, void *stream);

/*
 * The shuffling step for callers that replay it from a captured HIP graph.  A
 * captured launch repeats its arguments, so wash_shuffle in a graph would repeat
 * one step number and with it one mask and one set of permutations; Alg. 1
 * draws fresh ones at every iteration.  Here the kernel reads the step number
 * from device memory when it runs:
 *   step_dev   device uint64; its value when the kernel runs is the step of that
 *              launch (the low 32 bits are used: keep it below 2^32); must not
 *              overlap the buffers
 *   advance    1: *step_dev is incremented by one after the shuffle, on the same
 *              stream, so successive launches or replays walk through the steps;
 *              0: left alone (the caller updates it between replays)
 *   others     as for wash_shuffle_states
 * With *step_dev = s the result is bit-identical to wash_shuffle_states with
 * step = s.  As with the other shuffle entry points, a segment list seen for the
 * first time builds a device table (allocation + copy): make one call outside the
 * capture first.  A table that a capturing stream has used is kept until
 * wash_shutdown (replays read it), whatever other segment lists come later; call
 * wash_shutdown only once no graph that contains a shuffle will be replayed again.
 * Errors: as for wash_shuffle_states, plus WASH_EINVAL for step_dev = NULL or
 * advance not 0 or 1.  The value of *step_dev cannot be checked on the host.
 */
int wash_shuffle_device_step(float *const *buffers, uint32_t nbuffers, uint32_t N, uint64_t P,
                             const wash_segment *segs, uint32_t nsegs,
                             uint64_t seed, uint64_t *step_dev, int advance, int gap_stream,
                             uint64_t *selected_count, void *stream);

/*
 * Uniform average, Alg. 1 output line: out[g] = (1/N) sum_n params[n][g],
 * summed in fp64 in ascending n and rounded once to fp32.
 *   params  device, [N, P] fp32 (read only)      out  device, [P] fp32, must not overlap params
 * Errors: WASH_EINVAL for NULL pointers, N = 0 or > WASH_MAX_N, P = 0.
 */
int wash_average(const float *params, float *out, uint32_t N, uint64_t P, void *stream);

/*
 * PAPA's update, Eq. 1: params[n][g] <- alpha * params[n][g] + (1 - alpha) * mean[g]
 * for all n, where mean[g] is the average over n of the values BEFORE the
 * update; one pass, in place, arithmetic in fp64, rounded once to fp32.
 * alpha = 1 is the identity, alpha = 0 replaces every model by the consensus.
 *   params  device, [N, P] fp32, in place        alpha  any finite value (the paper uses ]0,1[)
 * Errors: WASH_EINVAL for NULL params, N = 0 or > WASH_MAX_N, P = 0, alpha NaN or infinite.
 */
int papa_ema(float *params, uint32_t N, uint64_t P, float alpha, void *stream);

/*
 * Distance to the consensus, the diagnostic behind Eq. 2, Eq. 5 and the
 * distance-to-consensus figures (which also look at slices of the parameter
 * vector): out[n] = sum over g in [g_begin, g_end) of (params[n][g] - mean[g])^2,
 * mean[g] = (1/N) sum_n params[n][g], everything in fp64.  The caller takes
 * sqrt / averages over n (the figures plot (1/N) sum_n sqrt(out[n])).  The
 * reduction has a fixed shape: the same input gives the same bits every time.
 *   params  device, [N, P] fp32 (read only)    out  device, N doubles (overwritten)
 *   g_begin <= g_end <= P   (an empty slice gives zeros)
 * The partial sums live in the workspace of the calling stream, so calls on
 * different streams do not interfere.
 * Errors: WASH_EINVAL for NULL pointers, N = 0 or > WASH_MAX_N, P = 0, a slice
 * outside [0, P]; WASH_EHIP if the scratch cannot be allocated or a launch fails.
 */
int wash_consensus_sqdist(const float *params, uint32_t N, uint64_t P,
                          uint64_t g_begin, uint64_t g_end, double *out, void *stream);

/*
 * wash_consensus_sqdist for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels, same result bit for bit; the partial sums go to
 * a fixed 1 MiB array in the library's device image instead of an allocated
 * buffer, so the call makes no hipMalloc / hipFree and calls no allocating
 * routine (the first call on a device looks up the array's address there).
 * Limits: N <= WASH_MAX_N and P <= 2^40, which is all the fixed array has to
 * cover (at most 4096 blocks x 32 partial sums); anything larger is WASH_EINVAL
 * as in wash_consensus_sqdist.  Every GPU the library runs on holds its own copy
 * of the array until the process ends.  All calls on one GPU share that copy:
 * two calls that overlap there (different streams) race on it and may return
 * wrong sums; calls on one stream are ordered and safe.  Nothing in the array
 * has to start at zero (every slot a launch reads, it has written first).
 */
int wash_consensus_sqdist_noalloc(const float *params, uint32_t N, uint64_t P,
                                  uint64_t g_begin, uint64_t g_end, double *out, void *stream);

/*
 * Weighted combination of the models: out[g] = sum_n weights[n] * params[n][g],
 * products and sum in fp64 in ascending n, rounded once to fp32.  Convex
 * weights give the interpolations studied in the appendix; a 0/1-over-k vector
 * gives a soup over a subset; weights 1/N give the uniform average up to the
 * rounding of 1/N (wash_average divides the sum instead).
 *   params   device, [N, P] fp32 (read only)    out  device, [P] fp32, must not overlap params
 *   weights  HOST array of N finite doubles, read before the call returns
 * Errors: WASH_EINVAL for NULL pointers, N = 0 or > WASH_MAX_N, P = 0, a
 * non-finite weight.
 */
int wash_weighted_average(const float *params, const double *weights, float *out,
                          uint32_t N, uint64_t P, void *stream);

/*
 * Layer-wise probabilities, Eq. 6 (host only): out[l] for l = 0 .. L-1.
 *   schedule 0  decreasing, p * (1 - l/(L-1))   (Eq. 6: first layer p, last layer 0)
 *   schedule 1  constant p
 *   schedule 2  increasing, p * l/(L-1)         (the appendix ablation)
 * L = 1 gives p for every schedule.  out: HOST array of L doubles.
 * Errors: WASH_EINVAL for p outside [0,1] or NaN, L = 0, unknown schedule, NULL out.
 */
int wash_layer_probs(double p, uint32_t L, int schedule, double *out);

/* Text for a status code (static storage, never NULL). */
const char *wash_strerror(int status);

/* Detail of the last error raised on the calling thread ("" if none). */
const char *wash_last_error_detail(void);

/*
 * Tuning knobs (process-wide, not part of the method: results never depend
 * on them).  Returns WASH_EINVAL for an unknown option or a value out of range.
 *   WASH_OPT_TILE_COORDS  coordinates scanned by one wavefront in wash_shuffle;
 *                         a multiple of 256 in [256, 65536], or 0 = choose by P, N and the probabilities
 *   WASH_OPT_STREAM_MIN_BYTES  from this population size N*P*4 on (default 256 MiB, the size of the
 *                         Infinity Cache) papa_ema and wash_average run in their streaming shape:
 *                         non-temporal accesses and a capped number of blocks per compute unit
 *   WASH_OPT_GAP_BLOCKS   1024-coordinate blocks walked by one wavefront in wash_shuffle_gap;
 *                         a power of two in [1, 64], or 0 = choose by P and p
 *   WASH_OPT_AVERAGE_CHUNKS  0 = wash_average chooses its kernel and launch shape from N and P;
 *                         1, 2, 4, 8 = force the kernel that reads the rows one after the other,
 *                         with that many 1024-coordinate chunks per block
 *   WASH_OPT_SHUFFLE_BLOCKS_PER_CU  cap on the blocks (of four wavefronts) of the gathering shuffle
 *                         kernel resident on one compute unit: 1 .. 20, or 0 = no cap
 *   WASH_OPT_DENSE        wash_shuffle has a second code path that streams whole rows through
 *                         on-chip memory instead of gathering single values (same results);
 *                         0 = use it inside segments whose probability is high enough for it
 *                         to be faster (p >= 0.08), 1 = never, 2 = wherever N * buffers <= 63
 */
#define WASH_OPT_TILE_COORDS 1
#define WASH_OPT_AVERAGE_CHUNKS 4
#define WASH_OPT_GAP_BLOCKS 3
#define WASH_OPT_STREAM_MIN_BYTES 2
#define WASH_OPT_DENSE 5
#define WASH_OPT_SHUFFLE_BLOCKS_PER_CU 6
int wash_set_option(int option, int64_t value);

/* Free the cached device tables of every device (waits for the devices). */
int wash_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* WASH_H */
