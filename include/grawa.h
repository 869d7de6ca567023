/*
 * grawa.h -- C ABI of the MI355X (gfx950) GRAWA distributed-update library.
 *
 * GRAWA (gradient-based weighted averaging) periodically pulls M data-parallel
 * workers toward a center model that is a weighted average of the workers, the
 * weights being inversely proportional to each worker's gradient norm.  This
 * library computes one such distributed phase for all workers that live on one
 * GPU, plus the local SGD step taken between phases.
 *
 * Notation.  K = number of workers (the paper's M); L = number of layers (the
 * paper's K); P = parameters per worker.  Worker k's flat parameter vector is
 * row k of x, its gradient is row k of g:
 *     x : float  [K][ldx]   device, updated in place
 *     g : float or bfloat16 [K][ldg]   device, never written
 * Rows are contiguous, ld* >= P counts elements, columns >= P are never touched.
 * A "layer" is any contiguous segment [offsets[l], offsets[l+1]) of the flat
 * vector chosen by the caller (one parameter tensor, or a module).
 *
 * Conventions for every call below.
 *  - All data pointers are DEVICE pointers unless the comment says "host".
 *  - The caller owns every buffer it passes.  The library allocates device
 *    memory only inside grawa_plan_create and frees it in grawa_plan_destroy.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue their kernels on it and return without synchronising; two
 *    calls that use the same plan must be ordered on one stream (the plan's
 *    workspace is shared).
 *  - Calls that take a plan run on the device the plan was created on (they
 *    switch to it and back); calls without a plan run on the caller's current
 *    device, which must own the buffers and the stream.
 *  - For full speed give x and g row pitches that are multiples of 1 KiB
 *    (256 fp32 elements): rows then start on cache-line boundaries and the
 *    kernels use streaming accesses.  Any legal pitch gives the same results.
 *  - Base pointers of x, g, center_out must be 16-byte aligned and ldx*4,
 *    ldg*sizeof(g element) must be multiples of 16; otherwise
 *    GRAWA_ERR_ALIGNMENT.  Layer offsets may be arbitrary.
 *  - Arguments are validated before anything is launched: a call that returns an
 *    error has launched nothing and changed nothing.
 *  - No exception crosses this boundary; the return code is the only error
 *    channel.  grawa_status_string turns it into text.
 *  - Parameters are fp32.  Gradients are fp32 or bf16 (bf16 values are used as
 *    stored, widened exactly).
 */
#ifndef GRAWA_H
#define GRAWA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GRAWA_OK = 0,
    GRAWA_ERR_INVALID_ARG = 1, /* null pointer, bad size, non-monotone offsets, lambda outside [0,1], non-finite scalar */
    GRAWA_ERR_ALIGNMENT = 2,   /* base pointer or leading dimension not 16-byte aligned */
    GRAWA_ERR_WORKSPACE = 3,   /* the plan could not get its device workspace */
    GRAWA_ERR_UNSUPPORTED = 4, /* a size or dtype the library does not handle (K > GRAWA_MAX_WORKERS, ...) */
    GRAWA_ERR_HIP = 5          /* a HIP runtime call or a kernel launch failed */
} grawa_status_t;

typedef enum { GRAWA_F32 = 0, GRAWA_BF16 = 1 } grawa_dtype_t;

/* Which scalar score a worker gets in the model-level variants. */
typedef enum {
    GRAWA_NORM_LAYERSUM = 0, /* MGRAWA, Sec. 5.1 eq. (3): A_k = sum over layers of ||G_layer||_F  */
    GRAWA_NORM_FLAT = 1      /* vanilla GRAWA, Sec. 4.3.1 eq. (2): A_k = ||flattened gradient||_2 */
} grawa_norm_mode_t;

#define GRAWA_MAX_WORKERS 1024

/* Bits of the plan's non-finite-score flag word (grawa_plan_nonfinite). */
#define GRAWA_NONFINITE_LAYER_SCORE 1u /* a per-(worker, layer) score A_k^l of eq. (5)-(6), or a running estimate of it, was +inf or NaN */
#define GRAWA_NONFINITE_MODEL_SCORE 2u /* a per-worker score A_k of eq. (2) or (3), or the sum of a worker's estimates, was +inf or NaN */

typedef struct grawa_plan grawa_plan_t; /* opaque */

/* Text for a status code (static storage, never NULL). */
const char *grawa_status_string(grawa_status_t s);

/*
 * Plan: the shape of one problem (K workers, P parameters, L layers) and the
 * device workspace for it -- the layer offsets, a map from fixed-size tiles of
 * the flat vector to layers (no tile crosses a layer boundary), per-tile partial
 * sums, and the K x L tables of squared norms, scores and weights.
 *   out                 host pointer that receives the plan
 *   layer_offsets_host  host array of L+1 values, [0] = 0, strictly increasing,
 *                       [L] = P; may be NULL only when L == 1
 * Uses the current HIP device; the plan must be used on that device.
 * Errors: INVALID_ARG (K < 1, P < 1, L < 1, L > P, bad offsets, out NULL),
 * UNSUPPORTED (K > GRAWA_MAX_WORKERS), WORKSPACE / HIP (allocation or copy failed).
 */
grawa_status_t grawa_plan_create(grawa_plan_t **out, int K, int64_t P, int L,
                                 const int64_t *layer_offsets_host);

/* Frees the plan and its workspace.  The caller must have synchronised the
 * streams that used it.  NULL is accepted. */
grawa_status_t grawa_plan_destroy(grawa_plan_t *plan);

/*
 * Gradient-norm scores, Sec. 5.2 eq. (5)-(6): norms_out[k][l] = ||g_k restricted
 * to layer l||_F, the Frobenius norm of worker k's accumulated gradient in layer
 * l.  Every gradient value is widened to fp64 before it is squared and all
 * sums are fp64 in a fixed order: squares are exact, nothing underflows or
 * overflows for any magnitude the gradient type can hold, and results are
 * bit-reproducible.  The tables handed back (norms, weights, estimates) are
 * float32: an entry whose exact value lies outside the float32 range is
 * rounded to 0 or +inf there, while the weights used inside the update are
 * formed from the fp64 scores.  norms_out: device float [K][L].
 */
grawa_status_t grawa_grad_norms(grawa_plan_t *plan, const void *g, int64_t ldg,
                                grawa_dtype_t g_dtype, float *norms_out, void *stream);

/*
 * One model-level distributed phase (Sec. 4.3.1 and Sec. 5.1, the body of the
 * "if" in Algorithm 1):
 *   A_k     score of worker k from g, per `mode` (eq. (3) or eq. (2))
 *   beta_k  = (1/A_k) / sum_j (1/A_j)                            (eq. (4))
 *   x_C     = sum_k beta_k x_k
 *   x_k    <- (1 - lambda) x_k + lambda x_C   for every k, from the pre-pull x
 * lambda must be finite and in [0, 1].  center_out (float [P]) receives x_C if
 * not NULL; weights_out (float [K]) receives beta if not NULL.
 * Zero scores: if any A_k is exactly 0 those workers share the weight equally
 * and the rest get 0 (the limit A -> 0+); +inf gives weight 0; NaN propagates.
 */
grawa_status_t grawa_mgrawa_update(grawa_plan_t *plan, float *x, int64_t ldx, const void *g,
                                   int64_t ldg, grawa_dtype_t g_dtype, grawa_norm_mode_t mode,
                                   float lambda, float *center_out, float *weights_out,
                                   void *stream);

/*
 * One layer-level distributed phase (Sec. 5.2 eqs. (5)-(7), the body of the
 * "if" in Algorithm 2): as above, but every layer l has its own scores
 * A_k^l = ||G_k^l||_F and its own weights beta_k^l normalised over the workers,
 * and the center is the concatenation of the per-layer weighted averages.
 * weights_out: float [K][L] or NULL.
 */
grawa_status_t grawa_lgrawa_update(grawa_plan_t *plan, float *x, int64_t ldx, const void *g,
                                   int64_t ldg, grawa_dtype_t g_dtype, float lambda,
                                   float *center_out, float *weights_out, void *stream);

/*
 * Non-finite scores.  The paper does not say what a worker with an infinite or
 * undefined gradient norm should get; by the weight formula a +inf score gives
 * weight 0 and a NaN score makes its whole group of weights NaN (see above).
 * Every call that turns scores into weights (the update calls, grawa_grad_norms,
 * the Local-GRAWA communication) also records the event in a flag word in the
 * plan's device workspace: GRAWA_NONFINITE_* bits, set on the device, sticky.
 * grawa_plan_nonfinite waits for `stream`, copies the word to *flags_host (host
 * pointer) and, if clear != 0, enqueues a kernel on `stream` that zeroes it.  It
 * synchronises, so it is a polling call for the host, not for a captured graph.
 */
grawa_status_t grawa_plan_nonfinite(grawa_plan_t *plan, unsigned *flags_host, int clear, void *stream);

/*
 * Center and pull with weights supplied by the caller (the display after eq. (2);
 * eq. (7) when per_layer != 0).  weights: device float [K] (per_layer == 0) or
 * [K][L] (per_layer != 0); they are used as given, not renormalised.
 */
grawa_status_t grawa_center_pull(grawa_plan_t *plan, float *x, int64_t ldx, const float *weights,
                                 int per_layer, float lambda, float *center_out, void *stream);

/*
 * Local SGD step of Algorithms 1 and 2: x_k <- x_k - lr * g_k for every worker.
 * Needs no plan.  lr must be finite.  K <= 65535 and P < 2^32 (UNSUPPORTED
 * beyond); the same limits hold for the other plan-less local steps below.
 */
grawa_status_t grawa_local_sgd(float *x, int64_t ldx, const void *g, int64_t ldg,
                               grawa_dtype_t g_dtype, int K, int64_t P, float lr, void *stream);

/*
 * Local SGD step fused into the distributed phase, in the order of Algorithms 1
 * and 2 (SGD step first, then the phase):
 *   x'_k = x_k - lr * gs_k ;  x_C = sum_k beta_k x'_k ;  x_k <- (1-lambda) x'_k + lambda x_C
 * with beta from the scores of g (as in the calls above).  g_sgd may be the same
 * array as g (the local-gradient variant of Appendix G) or a different one; it
 * has the same dtype as g and its own leading dimension.
 */
grawa_status_t grawa_mgrawa_update_sgd(grawa_plan_t *plan, float *x, int64_t ldx, const void *g,
                                       int64_t ldg, grawa_dtype_t g_dtype, grawa_norm_mode_t mode,
                                       float lambda, const void *g_sgd, int64_t ldg_sgd, float lr,
                                       float *center_out, float *weights_out, void *stream);

grawa_status_t grawa_lgrawa_update_sgd(grawa_plan_t *plan, float *x, int64_t ldx, const void *g,
                                       int64_t ldg, grawa_dtype_t g_dtype, float lambda,
                                       const void *g_sgd, int64_t ldg_sgd, float lr,
                                       float *center_out, float *weights_out, void *stream);

/*
 * Local SGD step followed by the proximity step of Algorithms 1 and 2 (the line
 * marked "Prox."), for every worker:
 *   x_k <- x_k - lr * g_k ;   x_k <- (1 - mu/tau) x_k + (mu/tau) x_C
 * center: device float [P], the center stored by the last distributed phase
 * (the center_out of an update call); it is read once per column for all K
 * workers.  mu is the proximity strength, tau the communication period;
 * 0 <= mu <= tau, tau > 0.  Needs no plan.
 */
grawa_status_t grawa_local_sgd_prox(float *x, int64_t ldx, const void *g, int64_t ldg,
                                    grawa_dtype_t g_dtype, int K, int64_t P, float lr,
                                    const float *center, float mu, float tau, void *stream);

/*
 * Local MGRAWA / LGRAWA (Appendix G): the gradient-norm scores come from the local
 * optimizer's own gradients instead of a separate accumulation phase.
 *
 * grawa_local_step_scored: one local step of all K workers, in the order of the
 * appendix's algorithm, with the gradient read ONCE:
 *   g_cur[k][l] = ||g_k restricted to layer l||_F
 *   t <- t + 1 ;  g_mvg <- gamma g_mvg + (1 - gamma) g_cur          (kept in the plan, fp64)
 *   x_k <- x_k - lr g_k ;  if center != NULL: x_k <- (1 - mu/tau) x_k + (mu/tau) center
 * 0 < gamma < 1, and gamma must not change between two communications
 * (INVALID_ARG).
 *
 * grawa_local_lgrawa_update / grawa_local_mgrawa_update: the communication step:
 *   g_est = gamma g_mvg / (1 - gamma^t)            (as printed, leading gamma included)
 *   weights from g_est: per layer (eq. (7)), or per model from the sum of a
 *   worker's layer estimates (eq. (3)-(4)); center and pull as in the calls above;
 *   then g_mvg <- 0, t <- 0.
 * est_out (device float [K][L] or NULL) receives g_est, weights_out the weights
 * ([K][L] or [K]).  INVALID_ARG if no local step was taken since the last
 * communication.  The step counter t lives in the plan's device workspace: it is
 * advanced by the scored step's own kernels and read by the communication's, so
 * these calls may be recorded into a HIP graph and replayed (every replay counts
 * its steps again).  The host keeps a mirror of t as of the last enqueued call
 * for the two INVALID_ARG checks above only; a replayed communication that finds
 * t = 0 on the device takes all estimates as zero (plain average).  All calls on
 * one plan must come from one thread, in stream order.
 *
 * grawa_local_scores_reset: g_mvg <- 0, t <- 0 without a communication.
 */
grawa_status_t grawa_local_step_scored(grawa_plan_t *plan, float *x, int64_t ldx, const void *g,
                                       int64_t ldg, grawa_dtype_t g_dtype, float lr,
                                       const float *center, float mu, float tau, float gamma,
                                       void *stream);
grawa_status_t grawa_local_lgrawa_update(grawa_plan_t *plan, float *x, int64_t ldx, float lambda,
                                         float *center_out, float *weights_out, float *est_out,
                                         void *stream);
grawa_status_t grawa_local_mgrawa_update(grawa_plan_t *plan, float *x, int64_t ldx, float lambda,
                                         float *center_out, float *weights_out, float *est_out,
                                         void *stream);
grawa_status_t grawa_local_scores_reset(grawa_plan_t *plan, void *stream);

/*
 * Local optimizer of the experiments (Appendix B.2.2: SGD with momentum, Nesterov
 * acceleration and weight decay), one step for every worker.  The paper names the
 * method without printing it; the form computed is
 *   d = g_k + weight_decay x_k ;  buf_k <- momentum buf_k + d ;
 *   x_k <- x_k - lr (d + momentum buf_k)
 * whose iterates are the look-ahead points of Nesterov's accelerated gradient.
 * buf: device float [K][ldb], the momentum buffer, updated in place; the caller
 * zeroes it before the first step and keeps it between steps.  buf and ldb obey
 * the rules of x and ldx (16-byte aligned base, ldb % 4 == 0, ldb >= P).
 * momentum >= 0, weight_decay >= 0, all finite.  Needs no plan.
 */
grawa_status_t grawa_local_nesterov(float *x, int64_t ldx, const void *g, int64_t ldg,
                                    grawa_dtype_t g_dtype, float *buf, int64_t ldb, int K, int64_t P,
                                    float lr, float momentum, float weight_decay, void *stream);

/*
 * Distributed phase of the two competing center rules of Appendix F, on the same
 * K x P layout and with the same pull  x_k <- (1-lambda) x_k + lambda x_C.
 *
 * grawa_easgd_update: x_a = (1/K) sum_k x_k ;  x_C <- (1 - rho) x_C + rho x_a
 *   (the center is averaged over workers and over time; the line printed in the
 *   appendix has x_a on both sides and is read with the previous center on the
 *   left).  center: device float [P], 16-byte aligned, REQUIRED: previous center on
 *   entry, new center on return.  0 <= rho <= 1.
 *
 * grawa_lsgd_update: x_C = x_k of the worker with the smallest loss (the first
 *   one on ties).  losses: device float [K].  center_out (device float [P] or
 *   NULL) receives x_C, leader_out (device int32 or NULL) the leader's index.
 */
grawa_status_t grawa_easgd_update(grawa_plan_t *plan, float *x, int64_t ldx, float lambda, float rho,
                                  float *center, void *stream);
grawa_status_t grawa_lsgd_update(grawa_plan_t *plan, float *x, int64_t ldx, const float *losses,
                                 float lambda, float *center_out, int *leader_out, void *stream);

/*
 * grawa_lgrawa_update without any allocation, for callers that cannot call
 * hipMalloc: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  It needs no plan.  The workspace a plan would own (tile
 * map, cell map, per-tile partial sums, the K x L tables) lives in a fixed
 * 32 MiB array inside the library's device image, one copy per GPU, held until
 * the process ends; the maps are built by two small kernels from layer offsets
 * that are already in DEVICE memory.  The call enqueues kernels on `stream` and
 * nothing else (no hipMalloc / hipFree / memset / copy, no synchronisation), and
 * gives bit for bit what grawa_lgrawa_update gives for the same inputs.
 *   layer_offsets_dev   device int64 [L+1], 8-byte aligned: [0] = 0, strictly
 *                       increasing, [L] = P.  They cannot be checked from the
 *                       host: offsets that break the rule give meaningless
 *                       values, but every access stays inside the buffers.
 *   x, g, lambda, center_out, weights_out: as in grawa_lgrawa_update.
 * Limits: K <= GRAWA_MAX_WORKERS, and the workspace must fit the array:
 *   4*ceil(P/256) + (16 + 8K)*(P/T + L + 1) + 16*K*L + 4K + 4L bytes (each part
 *   rounded up to 256) <= 32 MiB, T the tile length a plan would pick (2048 ..
 *   16384); the largest benchmark configuration (P = 354 M, K = 8) needs 7 MiB.
 *   Beyond that:
 *   GRAWA_ERR_UNSUPPORTED, nothing launched.
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU
 * (two streams, two threads) race and must be ordered by the caller.  The
 * first call on a device looks up the array's address (no allocation, but do
 * not make it while a capture is in progress on that device).
 */
grawa_status_t grawa_lgrawa_update_static(int K, int64_t P, int L, const int64_t *layer_offsets_dev,
                                          float *x, int64_t ldx, const void *g, int64_t ldg,
                                          grawa_dtype_t g_dtype, float lambda, float *center_out,
                                          float *weights_out, void *stream);

/*
 * Measurement aids (not part of the method).
 *
 * grawa_plan_profile: with enable != 0 the plan attaches a start and a stop
 * HIP event to the launch of the gradient-norm kernel and of the center+pull
 * kernel of every later update call (the events time the dispatch itself and
 * queue nothing extra on the stream; up to 4096 calls, then it stops
 * recording).  With enable == 0 recording stops.  Either way the counters are
 * reset.
 *
 * grawa_plan_profile_read: the caller must have synchronised the stream.
 * Returns the number of recorded calls in *n_calls and the summed durations in
 * milliseconds of the two kernels (host pointers; any may be NULL).
 *
 * grawa_plan_profile_read_call: the same for recorded call i alone
 * (0 <= i < n_calls, else INVALID_ARG), plus in *span_ms the time from the start
 * of its gradient-norm kernel to the end of its center+pull kernel, i.e. the
 * whole update on the device (for a call without a norm pass: the pull alone).
 *
 * grawa_stream_copy: dst[i] = src[i] for nbytes bytes (multiple of 16, both
 * pointers 16-byte aligned) with the same 128-bit access pattern as the update
 * kernels; a plain copy of known size used to calibrate hardware counters and
 * to measure the attainable HBM bandwidth of the machine.
 */
grawa_status_t grawa_plan_profile(grawa_plan_t *plan, int enable);
grawa_status_t grawa_plan_profile_read(grawa_plan_t *plan, int *n_calls, double *norm_ms,
                                       double *pull_ms);
grawa_status_t grawa_plan_profile_read_call(grawa_plan_t *plan, int i, double *norm_ms, double *pull_ms,
                                            double *span_ms);
grawa_status_t grawa_stream_copy(void *dst, const void *src, int64_t nbytes, void *stream);

/* Number of tiles the plan cut the flat vector into, and the tile length in
 * elements (host-side queries; for tests and the byte model). */
grawa_status_t grawa_plan_info(const grawa_plan_t *plan, int64_t *n_tiles, int *tile_elems);

#ifdef __cplusplus
}
#endif
#endif /* GRAWA_H */
