// Gradient norms and weights of the GRAWA update (gfx950, wave64).
//
//   k_sumsq            per (tile, worker) sum of squares of the gradient   [eq. (3), (5)]
//   k_finalize_layers  per layer: tile partials -> ||G||_F^2, ||G||_F, per-layer weights
//                      (optionally the running estimate of Appendix G)     [eq. (5)-(7)]
//   k_finalize_model   per worker: model score, model-level weights        [eq. (2)-(4)]
//   k_local_weights    weights from the running norm estimate              [App. G]
//   k_center_weights   EASGD (uniform) and LSGD (leader) weights           [App. F]
//
// The norm pass is a read-only stream: it runs fastest with several non-temporal loads per
// lane in flight and a capped occupancy.  Squares and sums are fp64 throughout, added in a
// fixed order (no atomics), so results are bit-reproducible.
#include "grawa_device.h"

// ---------------------------------------------------------------------------------
// gradient norms: per-tile sums of squares
// ---------------------------------------------------------------------------------

// grid (n_tiles, K), block 256.  partials[k][tile] = sum over the tile of g[k][i]^2.
// Each lane issues 8 independent 8-byte streaming loads per trip and keeps one accumulator
// per load; with the occupancy capped at 4 waves per SIMD this shape measured fastest for a
// read-only stream on this part (7.3-7.4 TB/s; 16-byte loads at full occupancy 6.9-7.0).
// Every value is widened to fp64 before it is squared and every sum is fp64: the squares are
// exact, so gradients of any magnitude the input type holds (1e-38 .. 3e38) give the same
// norms as a float64 evaluation up to the order of the additions.  The pass needs under a
// fifth of the fp64 rate at full HBM speed, so this costs no time.
#define GRAWA_SUMSQ_U 8
template <typename GT>
__global__ __launch_bounds__(GRAWA_BLOCK) __attribute__((amdgpu_waves_per_eu(1, 4))) void k_sumsq(
    const GT *__restrict__ g, int64_t ldg, const GrawaTile *__restrict__ tiles, int64_t n_tiles,
    double *__restrict__ partials)
{
    constexpr int V = Grad<GT>::VEC8;
    const GrawaTile t = tiles[blockIdx.x];
    const int k = blockIdx.y;
    const GT *row = g + (int64_t)k * ldg;
    const int tid = threadIdx.x;

    const int64_t a = t.start, b = t.start + t.len;
    int64_t a_al = (a + V - 1) / V * V;
    if (a_al > b) a_al = b;
    int64_t b_al = b / V * V;
    if (b_al < a_al) b_al = a_al;

    double acc[GRAWA_SUMSQ_U];
#pragma unroll
    for (int u = 0; u < GRAWA_SUMSQ_U; ++u) acc[u] = 0.0;

    // unaligned head (< V elements) on the first lanes, tail on the lanes of the second wave
    if (tid < (int)(a_al - a)) {
        acc[0] = sq_add(Grad<GT>::one(row + a + tid), 0.0);
    }
    if (tid >= GRAWA_WAVE && tid - GRAWA_WAVE < (int)(b - b_al)) {
        acc[1] = sq_add(Grad<GT>::one(row + b_al + (tid - GRAWA_WAVE)), 0.0);
    }

    // Body: all loads of a trip are issued before any is used.  Full trips need no bounds
    // checks; the last, partial trip loads a clamped (valid) address and discards the value.
    const int nvec = (int)((b_al - a_al) / V);
    const GT *body = row + a_al;
    typename Grad<GT>::Vec8 q[GRAWA_SUMSQ_U];
    int j0 = tid;
    for (; j0 + (GRAWA_SUMSQ_U - 1) * GRAWA_BLOCK < nvec; j0 += GRAWA_SUMSQ_U * GRAWA_BLOCK) {
#pragma unroll
        for (int u = 0; u < GRAWA_SUMSQ_U; ++u) q[u] = Grad<GT>::load8(body + (int64_t)(j0 + u * GRAWA_BLOCK) * V);
        __builtin_amdgcn_sched_barrier(0); // keep the arithmetic from being hoisted between the loads
#pragma unroll
        for (int u = 0; u < GRAWA_SUMSQ_U; ++u) acc[u] = Grad<GT>::sumsq8(q[u], acc[u]);
    }
    if (j0 < nvec) {
#pragma unroll
        for (int u = 0; u < GRAWA_SUMSQ_U; ++u) {
            const int j = j0 + u * GRAWA_BLOCK;
            q[u] = Grad<GT>::load8(body + (int64_t)(j < nvec ? j : j0) * V);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < GRAWA_SUMSQ_U; ++u) {
            const double r = Grad<GT>::sumsq8(q[u], 0.0);
            acc[u] += (j0 + u * GRAWA_BLOCK < nvec) ? r : 0.0;
        }
    }

    __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
    double lane = 0.0;
#pragma unroll
    for (int u = 0; u < GRAWA_SUMSQ_U; ++u) lane += acc[u];
    const double total = block_sum(lane, sm);
    if (tid == 0) partials[(int64_t)k * n_tiles + blockIdx.x] = total;
}

// ---------------------------------------------------------------------------------
// weights
// ---------------------------------------------------------------------------------

#define GRAWA_FIN_BLOCK 1024
#define GRAWA_FIN_WAVES (GRAWA_FIN_BLOCK / GRAWA_WAVE)

// Weights of one group of K scores held in LDS (sA[k], k < K): beta_k proportional to
// 1/A_k, summing to one, evaluated as (A_min/A_k) / sum_j (A_min/A_j) so that nothing
// overflows.  Scores of exactly zero share the weight equally and take all of it (the
// limit A -> 0+).  Called by ONE full wave (all 64 lanes); lanes stride over the workers.
// A score that is +inf or NaN sets `bit` in the plan's flag word (flags may be null).
__device__ __forceinline__ void group_weights(const double *sA, int K, float *beta, int64_t stride,
                                              float *beta_user, unsigned *flags, unsigned bit)
{
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    double mn = INFINITY, nz = 0.0, bad = 0.0;
    for (int k = lane; k < K; k += GRAWA_WAVE) {
        const double a = sA[k];
        mn = fmin(mn, a);
        nz += (a == 0.0) ? 1.0 : 0.0;
        bad += isfinite(a) ? 0.0 : 1.0;
    }
    const double a_min = wave_min(mn);
    const double n_zero = wave_sum(nz);
    if (flags && wave_sum(bad) > 0.0 && lane == 0) atomicOr(flags, bit);
    double z = 0.0;
    if (n_zero == 0.0)
        for (int k = lane; k < K; k += GRAWA_WAVE) z += a_min / sA[k];
    const double zsum = wave_sum(z);
    for (int k = lane; k < K; k += GRAWA_WAVE) {
        const double a = sA[k];
        double b;
        if (n_zero > 0.0)
            b = (a == 0.0) ? 1.0 / n_zero : 0.0;
        else
            b = (a_min / a) / zsum;
        beta[(int64_t)k * stride] = (float)b;
        if (beta_user) beta_user[(int64_t)k * stride] = (float)b;
    }
}

// Sum of p[t0 + first], p[t0 + first + step], ... below t1 over the lanes of one wave, four
// independent loads in flight per lane; every lane gets the total.
__device__ __forceinline__ double wave_strided_sum(const double *__restrict__ p, int t0, int t1, int first,
                                                   int step)
{
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int t = t0 + first;
    for (; t + 3 * step < t1; t += 4 * step) {
        s0 += p[t];
        s1 += p[t + step];
        s2 += p[t + 2 * step];
        s3 += p[t + 3 * step];
    }
    for (; t < t1; t += step) s0 += p[t];
    return wave_sum((s0 + s1) + (s2 + s3));
}

// grid L, block 1024 (16 waves).  Block l adds the tile partials of layer l for every worker
// and turns the K layer norms into the K per-layer weights.  With K >= 16 every wave takes
// workers w, w+16, ...; with fewer workers 16/K waves share one worker's tiles and their
// results are added in wave order.  All sums are fp64 in a fixed order (no atomics).
__global__ __launch_bounds__(GRAWA_FIN_BLOCK) void k_finalize_layers(
    const double *__restrict__ partials, int64_t n_tiles, const int32_t *__restrict__ layer_tile0,
    int K, int L, double *__restrict__ S, float *__restrict__ A, float *__restrict__ A_user,
    float *__restrict__ beta, float *__restrict__ beta_user, double *__restrict__ mvg, double gamma,
    int64_t *__restrict__ local_t, unsigned *__restrict__ flags)
{
    __shared__ double sA[GRAWA_MAX_WORKERS];
    __shared__ double sw[GRAWA_FIN_WAVES];
    const int l = blockIdx.x;
    // One more local step has fed the running estimate (Appendix G: t <- t + 1).  The counter lives
    // on the device so that a recorded and replayed call still counts.
    if (mvg && l == 0 && threadIdx.x == 0) *local_t += 1;
    const int t0 = layer_tile0[l], t1 = layer_tile0[l + 1];
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    const int wave = threadIdx.x / GRAWA_WAVE;
    if (K >= GRAWA_FIN_WAVES) {
        for (int k = wave; k < K; k += GRAWA_FIN_WAVES) {
            const double s = wave_strided_sum(partials + (int64_t)k * n_tiles, t0, t1, lane, GRAWA_WAVE);
            if (lane == 0) sA[k] = s;
        }
        __syncthreads();
    } else {
        const int share = GRAWA_FIN_WAVES / K; // waves per worker
        const int k = wave % K, part = wave / K;
        double s = 0.0;
        if (part < share)
            s = wave_strided_sum(partials + (int64_t)k * n_tiles, t0, t1, part * GRAWA_WAVE + lane,
                                 share * GRAWA_WAVE);
        if (lane == 0) sw[wave] = s;
        __syncthreads();
        if ((int)threadIdx.x < K) {
            double tot = 0.0;
            for (int j = 0; j < share; ++j) tot += sw[threadIdx.x + j * K];
            sA[threadIdx.x] = tot;
        }
        __syncthreads();
    }
    // sA[k] holds the squared norm; publish it, replace it by the norm, then the weights
    for (int k = threadIdx.x; k < K; k += GRAWA_FIN_BLOCK) {
        const double s = sA[k];
        const double a = sqrt(s);
        S[(int64_t)k * L + l] = s;
        A[(int64_t)k * L + l] = (float)a;
        if (A_user) A_user[(int64_t)k * L + l] = (float)a;
        sA[k] = a;
        // running estimate of Appendix G: g_mvg <- gamma g_mvg + (1 - gamma) g_cur
        if (mvg) mvg[(int64_t)k * L + l] = gamma * mvg[(int64_t)k * L + l] + (1.0 - gamma) * a;
    }
    __syncthreads();
    if (wave == 0) group_weights(sA, K, beta + l, L, beta_user ? beta_user + l : nullptr, flags, GRAWA_NONFINITE_LAYER_SCORE);
}

// Weights from the running norm estimate g_est = gamma g_mvg / (1 - gamma^t) (Appendix G), t =
// the device-side count of local steps since the last communication.  per_layer: grid L, block
// l normalises column l over the workers (eq. (7)); otherwise grid 1: score of worker k is the
// sum of its layer estimates (eq. (3) applied to the estimates), then eq. (4).  est_user (float
// [K][L], may be null) receives g_est.  With t = 0 (no step was counted) the estimates are taken
// as zero, which the zero-norm rule turns into the plain average.
__global__ __launch_bounds__(GRAWA_FIN_BLOCK) void k_local_weights(const double *__restrict__ mvg, double gamma,
                                                                   const int64_t *__restrict__ local_t,
                                                                   int K, int L, int per_layer,
                                                                   float *__restrict__ beta,
                                                                   float *__restrict__ beta_user,
                                                                   float *__restrict__ est_user,
                                                                   unsigned *__restrict__ flags)
{
    __shared__ double sA[GRAWA_MAX_WORKERS];
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    const int wave = threadIdx.x / GRAWA_WAVE;
    const int64_t t = *local_t;
    const double scale = t > 0 ? gamma / (1.0 - pow(gamma, (double)t)) : 0.0;
    if (per_layer) {
        const int l = blockIdx.x;
        for (int k = threadIdx.x; k < K; k += GRAWA_FIN_BLOCK) {
            const double e = scale * mvg[(int64_t)k * L + l];
            sA[k] = e;
            if (est_user) est_user[(int64_t)k * L + l] = (float)e;
        }
        __syncthreads();
        if (wave == 0)
            group_weights(sA, K, beta + l, L, beta_user ? beta_user + l : nullptr, flags, GRAWA_NONFINITE_LAYER_SCORE);
    } else {
        for (int k = wave; k < K; k += GRAWA_FIN_WAVES) {
            double s = 0.0;
            for (int l = lane; l < L; l += GRAWA_WAVE) {
                const double e = scale * mvg[(int64_t)k * L + l];
                s += e;
                if (est_user) est_user[(int64_t)k * L + l] = (float)e;
            }
            s = wave_sum(s);
            if (lane == 0) sA[k] = s;
        }
        __syncthreads();
        if (wave == 0) group_weights(sA, K, beta, 1, beta_user, flags, GRAWA_NONFINITE_MODEL_SCORE);
    }
}

// g_mvg <- 0 and t <- 0 (after a communication, or an explicit reset).
__global__ __launch_bounds__(GRAWA_BLOCK) void k_zero_estimate(double *__restrict__ p, int64_t n,
                                                               int64_t *__restrict__ local_t)
{
    const int64_t i = (int64_t)blockIdx.x * GRAWA_BLOCK + threadIdx.x;
    if (i < n) p[i] = 0.0;
    if (i == 0) *local_t = 0;
}

// grid 1, block 1024.  Model-level score per worker from the [K][L] squared layer norms:
// mode 0: sum of the layer norms; mode 1: norm of the flattened gradient.  Then the K weights.
__global__ __launch_bounds__(GRAWA_FIN_BLOCK) void k_finalize_model(const double *__restrict__ S, int K,
                                                                    int L, int mode,
                                                                    float *__restrict__ beta,
                                                                    float *__restrict__ beta_user,
                                                                    unsigned *__restrict__ flags)
{
    __shared__ double sA[GRAWA_MAX_WORKERS];
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    const int wave = threadIdx.x / GRAWA_WAVE;
    for (int k = wave; k < K; k += GRAWA_FIN_WAVES) {
        const double *p = S + (int64_t)k * L;
        double s = 0.0;
        if (mode == GRAWA_NORM_LAYERSUM)
            for (int l = lane; l < L; l += GRAWA_WAVE) s += sqrt(p[l]);
        else
            for (int l = lane; l < L; l += GRAWA_WAVE) s += p[l];
        s = wave_sum(s);
        if (mode != GRAWA_NORM_LAYERSUM) s = sqrt(s);
        if (lane == 0) sA[k] = s;
    }
    __syncthreads();
    if (wave == 0) group_weights(sA, K, beta, 1, beta_user, flags, GRAWA_NONFINITE_MODEL_SCORE);
}

// flag word <- 0
__global__ void k_clear_flags(unsigned *__restrict__ flags)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *flags = 0u;
}

// Weights of the competing centers of Appendix F, written where the pull kernel reads its
// model-level weights.  loss == nullptr: EASGD, every worker 1/K.  Otherwise LSGD: weight 1 for
// the worker with the smallest loss (the first one on ties), 0 for the rest; its index goes to
// leader_out when given.  One thread: K is at most 1024.
__global__ void k_center_weights(const float *__restrict__ loss, int K, float *__restrict__ beta,
                                 float *__restrict__ beta_user, int *__restrict__ leader_out)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int best = -1;
    if (loss) {
        best = 0;
        for (int k = 1; k < K; ++k)
            if (loss[k] < loss[best]) best = k;
        if (leader_out) *leader_out = best;
    }
    for (int k = 0; k < K; ++k) {
        const float b = loss ? (k == best ? 1.f : 0.f) : 1.f / (float)K;
        beta[k] = b;
        if (beta_user) beta_user[k] = b;
    }
}

// ---------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------

// Kernels that are timed carry their own start/stop events (taken from the dispatch itself,
// so nothing extra is queued on the stream); both may be null.
hipError_t grawa_launch_sumsq(const grawa_plan *p, const void *g, int64_t ldg, grawa_dtype_t dt,
                              hipStream_t s, hipEvent_t e0, hipEvent_t e1)
{
    const dim3 grid((unsigned)p->n_tiles, (unsigned)p->K), block(GRAWA_BLOCK);
    if (dt == GRAWA_BF16)
        hipExtLaunchKernelGGL(k_sumsq<uint16_t>, grid, block, 0, s, e0, e1, 0, (const uint16_t *)g, ldg,
                              (const GrawaTile *)p->d_tiles, p->n_tiles, p->d_partials);
    else
        hipExtLaunchKernelGGL(k_sumsq<float>, grid, block, 0, s, e0, e1, 0, (const float *)g, ldg,
                              (const GrawaTile *)p->d_tiles, p->n_tiles, p->d_partials);
    return hipGetLastError();
}

// update_estimate != 0: the partials come from the local step (short-tile map) and the running
// norm estimate is updated with the new norms.
hipError_t grawa_launch_finalize_layers(const grawa_plan *p, float *norms_user, float *beta_user,
                                        hipStream_t s, int update_estimate, double gamma)
{
    k_finalize_layers<<<dim3((unsigned)p->L), dim3(GRAWA_FIN_BLOCK), 0, s>>>(
        p->d_partials, update_estimate ? p->n_rtiles : p->n_tiles,
        update_estimate ? p->d_layer_rtile0 : p->d_layer_tile0, p->K, p->L, p->d_S, p->d_A, norms_user,
        p->d_beta_layer, beta_user, update_estimate ? p->d_mvg : nullptr, gamma, p->d_local_t, p->d_flags);
    return hipGetLastError();
}

hipError_t grawa_launch_local_weights(const grawa_plan *p, double gamma, int per_layer, float *beta_user,
                                      float *est_user, hipStream_t s)
{
    k_local_weights<<<dim3(per_layer ? (unsigned)p->L : 1u), dim3(GRAWA_FIN_BLOCK), 0, s>>>(
        p->d_mvg, gamma, p->d_local_t, p->K, p->L, per_layer, per_layer ? p->d_beta_layer : p->d_beta_model,
        beta_user, est_user, p->d_flags);
    return hipGetLastError();
}

hipError_t grawa_launch_zero_estimate(const grawa_plan *p, hipStream_t s)
{
    const int64_t n = (int64_t)p->K * p->L;
    k_zero_estimate<<<dim3((unsigned)((n + GRAWA_BLOCK - 1) / GRAWA_BLOCK)), dim3(GRAWA_BLOCK), 0, s>>>(p->d_mvg, n,
                                                                                                    p->d_local_t);
    return hipGetLastError();
}

hipError_t grawa_launch_finalize_model(const grawa_plan *p, grawa_norm_mode_t mode, float *beta_user,
                                       hipStream_t s)
{
    k_finalize_model<<<dim3(1), dim3(GRAWA_FIN_BLOCK), 0, s>>>(p->d_S, p->K, p->L, (int)mode,
                                                          p->d_beta_model, beta_user, p->d_flags);
    return hipGetLastError();
}

hipError_t grawa_launch_clear_flags(const grawa_plan *p, hipStream_t s)
{
    k_clear_flags<<<dim3(1), dim3(GRAWA_WAVE), 0, s>>>(p->d_flags);
    return hipGetLastError();
}

hipError_t grawa_launch_center_weights(const grawa_plan *p, const float *loss, float *beta_user, int *leader_out,
                                       hipStream_t s)
{
    k_center_weights<<<dim3(1), dim3(GRAWA_WAVE), 0, s>>>(loss, p->K, p->d_beta_model, beta_user, leader_out);
    return hipGetLastError();
}
