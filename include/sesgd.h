/*
 * sesgd.h -- C ABI of the Shuffle-Exchange SGD (SESGD) step library for AMD gfx950.
 *
 * The library simulates n logical data-parallel workers as n rows of one packed,
 * multi-layer buffer in a single GPU's memory and performs, per training iteration,
 *   (1) the regrouping of the workers into n/group_size equal groups
 *       (Sec. 3.1 "Shuffle-Exchange"; Algorithm 1, the two regrouping steps),
 *   (2) each worker's local SGD/momentum step followed by the average of the locally
 *       updated parameters inside the worker's group
 *       (Sec. 3.2 "Gradient Correction", the SESGD update equation; Algorithm 1),
 *   (3) as a baseline, the fully synchronous Ring-SGD/DSGD step
 *       (Sec. 3.2, the DSGD equation; Sec. 2.2 for the all-reduce it stands for).
 *
 * Conventions shared by all calls
 *   - Plain C, no exceptions, no torch types.  Every function returns SE_OK (0) or a
 *     negative SE_ERR_* code.  Arguments are validated on the host before anything is
 *     launched: a validation error (every code but SE_ERR_HIP) means nothing was written or
 *     launched.  A call may issue several launches (layer ranges with unaligned edges, large
 *     groups); SE_ERR_HIP from a later launch leaves the earlier ones enqueued.
 *   - "device" pointers are HIP device addresses owned by the caller; "host" pointers are
 *     ordinary host memory.  The library never frees or keeps a caller's pointer.
 *   - Replica layout: params, grads and momentum each hold n rows; row i (worker i)
 *     starts at base + i*pitch elements, pitch = layer_offsets[num_layers].  A caller who
 *     wants padded rows appends a dummy last layer so that the last offset is the pitch.
 *   - layer_offsets is a HOST array of num_layers+1 non-decreasing element offsets with
 *     layer_offsets[0] == 0.  Groups are drawn once per iteration for the whole model, and
 *     the update is elementwise, so the result does not depend on where the layer
 *     boundaries fall; the offsets define the pitch and are validated.
 *   - The three buffers must not overlap.  params and momentum are updated in place.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  se_step and
 *     se_ring_step only enqueue work on it and return without synchronising.  They record
 *     kernel launches only (no memset), so they may be captured in a HIP graph; the first
 *     launch of each kernel variant on a device also sets a function attribute, so make one
 *     ordinary call with the same argument types before capturing.
 *   - Device memory of the library's own: reductions over more than 8 rows (se_ring_step and
 *     se_global_average with n > 8, group_size > 8) on large buffers run as pairs of launches
 *     that hand means or block sums over through a buffer the library allocates on first use,
 *     one per (device, stream) for up to 16 such pairs, at most 128 MiB each by default, grown
 *     on demand and kept until the process ends.  Steps on different streams never share a
 *     buffer.  While `stream` is being captured, or when no buffer can be had, the one-launch
 *     form runs instead; results are bit-identical either way.
 *   - fp32 arithmetic, round-to-nearest-even, denormals kept, with this fixed order per
 *     element e and group with members j_0 < j_1 < ... (ascending worker id):
 *         v'_j   = fma(mu, v_j, g_j)            (g_j if momentum == NULL)
 *         xhat_j = fma(-lr, v'_j, x_j)
 *         s      = the xhat_j added up in the library's fixed order: the members in ascending id
 *                  are cut into consecutive blocks of 8 (the last may be shorter), each block is
 *                  added up left to right, then the block sums are added up left to right
 *                  (up to 8 members: the plain left-to-right sum)
 *         x_j    = s * (1.0f / (float)group_size)  for every member;   v_j = v'_j
 *     The same order is used wherever rows are added up (mean gradient, global average).
 *     NaN/Inf propagate.
 */
#ifndef SESGD_H
#define SESGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SE_OK                  0
#define SE_ERR_ARG           (-1)  /* n<1, group_size<1, group_size>n, iter<0, num_layers<0, bad layer range or flags */
#define SE_ERR_DIVISIBILITY  (-2)  /* n % group_size != 0: the paper defines equal groups only */
#define SE_ERR_NULL          (-3)  /* a required pointer is NULL */
#define SE_ERR_LAYOUT        (-4)  /* offsets not monotone, offsets[0]!=0, buffers overlap, misaligned */
#define SE_ERR_UNSUPPORTED   (-5)  /* n > SE_MAX_WORKERS, or pitch >= 2^30 elements */
#define SE_ERR_HIP           (-6)  /* a HIP call failed; se_last_error() has the HIP string */

#define SE_MAX_WORKERS 64          /* one wavefront lane per worker in the plan generator */

/*
 * Regrouping for iteration `iter` (Sec. 3.1; Algorithm 1: "randomly generate new groups
 * depending on the seed", "enter a new group").  Every worker derives the same partition
 * from the shared seed (se_set_seed), so no message is exchanged.  The partition is a
 * pure function of (seed, n, iter): workers are ordered by a 32-bit hash of
 * (seed, iter, n, worker id), ties by id, and the order is cut into blocks of group_size.
 *   group_of [host, n ints, out]           group index in [0, n/group_size) of each worker
 *   members  [host, n ints, out, may be NULL] group-major; members[g*group_size + r] is the
 *                                           r-th smallest worker id of group g
 * Runs the device generator on the current device, synchronously (default stream).  Allocates
 * and frees a small device buffer on every call (the free synchronises the device): meant for
 * tests and set-up code; inside a training loop use se_plan_device or se_plan_noalloc.
 */
int se_plan(int n, int group_size, int64_t iter, int32_t *group_of, int32_t *members);

/*
 * se_plan for callers that cannot allocate device memory (code that must not call hipMalloc:
 * tight serving loops, harnesses that forbid it, set-up code next to a stream capture).  Same
 * arguments, same results and same error codes as se_plan, but the device-side staging of the
 * two result arrays lives in a 512-byte array that is part of the library's code object (one
 * copy per GPU, kept until the process ends) instead of a buffer allocated and freed per call.
 * Calls no hipMalloc / hipFree.  Limit: n <= SE_MAX_WORKERS (64); a larger n returns
 * SE_ERR_UNSUPPORTED and touches nothing.  Synchronous, default stream, current device.  All
 * calls on one GPU share that array: calls that overlap in time on the same GPU (from several
 * threads or processes' streams) race and must be serialised by the caller.
 */
int se_plan_noalloc(int n, int group_size, int64_t iter, int32_t *group_of, int32_t *members);

/* Same, asynchronous: both outputs are DEVICE arrays of n ints written on `stream`
 * (members_dev may be NULL).  Allocates nothing. */
int se_plan_device(int n, int group_size, int64_t iter, int32_t *group_of_dev,
                   int32_t *members_dev, void *stream);

/*
 * One SESGD iteration over all layers in one launch (Sec. 3.2, the SESGD update equation;
 * Algorithm 1 loop body with the minibatch gradient already formed in `grads`).
 *   params   [device, n*pitch fp32, in/out]
 *   grads    [device, n*pitch fp32, in]
 *   momentum [device, n*pitch fp32, in/out]  may be NULL iff mu == 0: plain SGD, no
 *                                            momentum bytes are touched.  One buffer per
 *                                            worker; it is never averaged.
 *   group_size == 1 is local SGD without averaging; group_size == n is the full average:
 *   from identical starts it follows se_ring_step up to fp32 rounding (the two add different
 *   quantities up: x-hat here, gradients there): within 1e-6 of the layer maximum after the 10 to
 *   20 iterations of the library's test configurations with up to 64 workers; the difference
 *   random-walks with the iteration count and is not bounded for long runs.
 */
int se_step(float *params, const float *grads, float *momentum,
            const int64_t *layer_offsets, int num_layers,
            int n, int group_size, int64_t iter, float lr, float mu, void *stream);

/* Same with gradients stored as bfloat16 bit patterns (uint16); widening to fp32 is exact. */
int se_step_bf16g(float *params, const uint16_t *grads_bf16, float *momentum,
                  const int64_t *layer_offsets, int num_layers,
                  int n, int group_size, int64_t iter, float lr, float mu, void *stream);

/*
 * One Ring-SGD / DSGD iteration (Sec. 3.2, the DSGD equation): the mean gradient over all
 * n workers, gbar = (g_0, g_1, ..., g_{n-1} added up in the fixed order above) * (1.0f/(float)n), then on
 * every worker v_i = fma(mu, v_i, gbar) (gbar if momentum == NULL), x_i = fma(-lr, v_i, x_i).
 * Same buffers and layout as se_step.
 */
int se_ring_step(float *params, const float *grads, float *momentum,
                 const int64_t *layer_offsets, int num_layers,
                 int n, float lr, float mu, void *stream);

int se_ring_step_bf16g(float *params, const uint16_t *grads_bf16, float *momentum,
                       const int64_t *layer_offsets, int num_layers,
                       int n, float lr, float mu, void *stream);

/*
 * General form of the step.
 *   grads_are_bf16  0: grads points at fp32, else at bfloat16 bit patterns
 *   first_layer, last_layer   only columns layer_offsets[first_layer] .. layer_offsets[last_layer]
 *                   of every row are stepped (0 <= first_layer <= last_layer <= num_layers).
 *                   The paper sends layer l while backward computes layer l-1 (Sec. 2.1); a
 *                   caller reproduces that schedule with one call per layer range.  The groups
 *                   depend on iter only, so stepping every layer once with the same iter equals
 *                   one se_step.
 *   weight_decay    (Sec. 4.1 lists 5e-4 / 1e-4) folded into the momentum update as the
 *                   decayed gradient d = fma(weight_decay, x, g); 0 means none (d = g).
 *   flags           0: the SESGD update (Sec. 3.2 "Gradient Correction").
 *                   SE_FLAG_GRAD_AVG: the variant the paper rejects (Sec. 3.2, the shuffle
 *                   applied directly to the DSGD equation): the gradients are averaged inside
 *                   the group, gbar = (g_j0, g_j1, ... in the fixed order) * (1.0f/(float)group_size), and every
 *                   member updates on its own with d = fma(weight_decay, x_j, gbar),
 *                   v_j = fma(mu, v_j, d), x_j = fma(-lr, v_j, x_j).  Replicas drift apart.
 *                   With group_size == n this is se_ring_step.
 * Local-SGD / Local-SESGD (Sec. 4.1 baselines: synchronise every second iteration) need no
 * flag: an iteration without synchronisation is a call with group_size == 1.
 */
#define SE_FLAG_GRAD_AVG 1u
int se_step_ex(float *params, const void *grads, int grads_are_bf16, float *momentum,
               const int64_t *layer_offsets, int num_layers, int first_layer, int last_layer,
               int n, int group_size, int64_t iter, float lr, float mu, float weight_decay,
               unsigned flags, void *stream);

/* Final global average (Algorithm 1, last line): every row of params becomes
 * (x_0, x_1, ..., x_{n-1} added up in the fixed order) * (1.0f/(float)n).  Reads and writes
 * params only. */
int se_global_average(float *params, const int64_t *layer_offsets, int num_layers, int n,
                      void *stream);

/*
 * Replica-consistency diagnostics in double precision (the quantity of the divergence equation
 * of Sec. 3.2 and of the parameter-consistency experiment of Sec. 4.2; xbar as in Sec. 3.3):
 *   out_dev[0] = sum over columns e and workers i of (x_i[e] - xbar[e])^2, xbar[e] = mean_i x_i[e]
 *   out_dev[1] = sum of all n*pitch parameters
 * out_dev is a DEVICE array of two doubles, 8-byte aligned, written on `stream` (cleared by the
 * call itself).  The summation order over columns is not fixed: results agree with a
 * sequential evaluation to about 1e-13 relative; identical replicas give exactly 0.
 */
int se_consensus(const float *params, const int64_t *layer_offsets, int num_layers, int n,
                 double *out_dev, void *stream);

/*
 * Host-only calculator of the paper's communication-time model, to set a simulated step beside
 * the paper's cluster setting.  For every layer of G bytes (element count from layer_offsets
 * times elem_bytes), a ring all-reduce over w workers costs 2 (w-1) (G/(w*bandwidth) + latency)
 * seconds and 2 (w-1) handshakes (Sec. 2.2); Ring-SGD uses w = n, SESGD with `groups` groups
 * uses w = n/groups (Sec. 3.1).  bandwidth in bytes/s, latency in seconds.  Any output pointer
 * may be NULL.  Touches no device.
 */
int se_comm_model(const int64_t *layer_offsets, int num_layers, int elem_bytes, int n, int groups,
                  double bandwidth, double latency, double *ring_seconds, double *sesgd_seconds,
                  int64_t *ring_handshakes, int64_t *sesgd_handshakes);

/*
 * Host-only helper for stepping a model in layer ranges while backward still runs (Sec. 2.1:
 * the last layer's gradients are ready first, and the exchange of one layer overlaps the
 * backward pass of the layers before it).  One se_step_ex call per layer pays a launch for
 * every small tensor (Sec. 2.3 counts the same cost in handshakes); this cuts the layers, back
 * to front, into consecutive ranges of at least min_elements elements each.  Layers are never
 * split; the front-most range takes what is left and may be smaller.
 *   first_layer [host, out, `capacity` ints]  first layer of each range in stepping order (back
 *                to front): range i covers layers [first_layer[i], end_i) with end_0 =
 *                num_layers and end_i = first_layer[i-1]; pass them to se_step_ex as
 *                first_layer / last_layer
 *   num_ranges  [host, out]  number of ranges (0 for a model without layers)
 * When `capacity` is too small, *num_ranges is set, first_layer is left alone and SE_ERR_ARG is
 * returned (num_layers entries always suffice).  Touches no device.
 */
int se_layer_buckets(const int64_t *layer_offsets, int num_layers, int64_t min_elements,
                     int32_t *first_layer, int capacity, int *num_ranges);

/* The shared random seed of Algorithm 1 (process-wide, default 0).  Read at call time by
 * se_plan, se_plan_device and se_step. */
int      se_set_seed(uint64_t seed);
uint64_t se_get_seed(void);

/* Recommended row pitch for P elements: P rounded up to a multiple of 1024 elements, so that
 * with a 4 KiB-aligned base every row starts 4 KiB aligned: the 128-bit path is taken and each
 * wavefront's 1 KiB piece of a row is 1 KiB aligned (measured on MI355X: 3-4 % more bandwidth
 * than rows that are only 128-byte aligned, 20-25 % more than rows that start anywhere else; such
 * rows still move 128 bits per lane as long as each starts on a 4-byte boundary).  Returns -1
 * for P < 0. */
int64_t se_pitch(int64_t P);

/* Bytes the method itself moves per call over `columns` elements per worker (reads + writes
 * of params, grads, momentum), the numerator of the achieved-bandwidth figure:
 * n*columns*(8 + grad bytes + 8 if momentum).  Pass the P real elements for the algorithmic
 * figure, the pitch for what a full-range launch touches. */
int64_t se_step_bytes(int64_t columns, int n, int grad_elem_bytes, int has_momentum);

/* Static description of an error code; for SE_ERR_HIP, se_last_error() returns the text of
 * the failing HIP call of the calling thread's most recent failure. */
const char *se_strerror(int code);
const char *se_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SESGD_H */
