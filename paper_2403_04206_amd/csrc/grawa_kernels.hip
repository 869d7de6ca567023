// HIP kernels of the GRAWA distributed update for gfx950 (MI355X), wave64.
//
// The update is a streaming computation: every parameter and gradient element is read
// once per pass and there is no reuse, so each kernel is nothing but global loads and
// stores kept in flight.  There is no dense contraction here and therefore no matrix-core
// code.  Two measured facts shape the kernels:
//   * read-only streams (the norm pass) run fastest with 128-bit non-temporal loads, several
//     per lane;
//   * the read-modify-write pass over K far-apart rows runs fastest when a wave touches one
//     aligned 256-byte piece of every row (one 32-bit element per lane per row) and the
//     blocks are small and many, again with non-temporal accesses -- provided every row
//     starts on a 128-byte boundary, so that no cache line is written in two parts.
//
//   k_sumsq            per (tile, worker) sum of squares of the gradient   [eq. (3), (5)]
//   k_finalize_layers  per layer: tile partials -> ||G||_F^2, ||G||_F, per-layer weights
//                                                                          [eq. (5)-(7)]
//   k_finalize_model   per worker: model score, model-level weights        [eq. (2)-(4)]
//   k_center_pull      x_C = sum_k beta_k x_k ; x_k <- x_k + lambda (x_C - x_k), with the
//                      local SGD step x_k - lr g_k optionally applied on the way in
//                                                   [display after eq. (2); Alg. 1, 2]
//   k_local_sgd        x_k <- x_k - lr g_k                                 [Alg. 1, 2]
//   k_nesterov         SGD with Nesterov momentum and weight decay         [App. B.2.2]
//   k_center_weights   EASGD (uniform) and LSGD (leader) weights           [App. F]
#include <hip/hip_ext.h>

#include "grawa_internal.h"

#define GRAWA_BLOCK 256
#define GRAWA_WAVE 64

// ---------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_one(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Move a double between lanes with a DPP control word (both 32-bit halves).
template <int CTRL> __device__ __forceinline__ double dpp_move_f64(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes of a wave; every lane gets the total.  Within a row of 16 lanes:
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror; across the four
// rows: two butterfly exchanges.
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_move_f64<0xB1>(v);  // lane ^ 1
    v += dpp_move_f64<0x4E>(v);  // lane ^ 2
    v += dpp_move_f64<0x141>(v); // other quad of the half row
    v += dpp_move_f64<0x140>(v); // other half of the row
    v += __shfl_xor(v, 16, GRAWA_WAVE);
    v += __shfl_xor(v, 32, GRAWA_WAVE);
    return v;
}

__device__ __forceinline__ double wave_min(double v)
{
    for (int m = 1; m < GRAWA_WAVE; m <<= 1) v = fmin(v, __shfl_xor(v, m, GRAWA_WAVE));
    return v;
}

// Sum over a 256-thread block through LDS; every thread gets the result.  `sm` holds one
// double per wave.
__device__ __forceinline__ double block_sum(double v, double *sm)
{
    v = wave_sum(v);
    const int w = threadIdx.x / GRAWA_WAVE;
    __syncthreads();
    if ((threadIdx.x & (GRAWA_WAVE - 1)) == 0) sm[w] = v;
    __syncthreads();
    double t = 0.0;
    for (int i = 0; i < GRAWA_BLOCK / GRAWA_WAVE; ++i) t += sm[i];
    return t;
}

typedef float v2f __attribute__((ext_vector_type(2)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Global-memory accessors for the one-element-per-lane kernels.  An address is a wave-uniform
// 64-bit base plus a 32-bit lane byte offset; the base is pinned in a scalar register pair so
// that the access is issued in that form instead of with a 64-bit address computed per lane.
// NT = streaming (non-temporal) access.
#define GRAWA_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ uint64_t uniform_base(const void *p)
{
    uint64_t a = reinterpret_cast<uint64_t>(p);
    asm volatile("" : "+s"(a));
    return a;
}
// A float read through the scalar unit from memory this kernel never writes.
__device__ __forceinline__ float ld_uniform_f32(uint64_t base, int64_t index)
{
    return ((const __attribute__((address_space(4))) float *)base)[index];
}
template <bool NT, typename T> __device__ __forceinline__ T ld_lane(uint64_t base, unsigned byte_off)
{
    const GRAWA_GLOBAL T *p = (const GRAWA_GLOBAL T *)(base + byte_off);
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT, typename T> __device__ __forceinline__ void st_lane(uint64_t base, unsigned byte_off, T v)
{
    GRAWA_GLOBAL T *p = (GRAWA_GLOBAL T *)(base + byte_off);
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Gradient element access.  VEC8 = elements per 8-byte load (norm pass).
template <typename GT> struct Grad;

template <> struct Grad<float> {
    static constexpr int VEC8 = 2;
    static __device__ __forceinline__ float one(const float *p) { return *p; }
    template <bool NT> static __device__ __forceinline__ float lane(uint64_t base, unsigned off)
    {
        return ld_lane<NT, float>(base, off);
    }
    // 8 bytes (2 floats) at p, 8-byte aligned, streaming load; and their squares added to acc
    typedef v2f Vec8;
    static __device__ __forceinline__ Vec8 load8(const float *p)
    {
        return __builtin_nontemporal_load(reinterpret_cast<const v2f *>(p));
    }
    static __device__ __forceinline__ float sumsq8(Vec8 q, float acc)
    {
        acc = fmaf(q.x, q.x, acc);
        acc = fmaf(q.y, q.y, acc);
        return acc;
    }
};

template <> struct Grad<uint16_t> { // bfloat16 bit patterns
    static constexpr int VEC8 = 4;
    static __device__ __forceinline__ float one(const uint16_t *p) { return bf16_one(*p); }
    template <bool NT> static __device__ __forceinline__ float lane(uint64_t base, unsigned off)
    {
        return bf16_one(ld_lane<NT, uint16_t>(base, off));
    }
    // 8 bytes (4 bf16) at p, 8-byte aligned, streaming load; and their squares added to acc
    typedef v2u Vec8;
    static __device__ __forceinline__ Vec8 load8(const uint16_t *p)
    {
        return __builtin_nontemporal_load(reinterpret_cast<const v2u *>(p));
    }
    static __device__ __forceinline__ float sumsq8(Vec8 q, float acc)
    {
        float a;
        a = bf16_lo(q.x); acc = fmaf(a, a, acc);
        a = bf16_hi(q.x); acc = fmaf(a, a, acc);
        a = bf16_lo(q.y); acc = fmaf(a, a, acc);
        a = bf16_hi(q.y); acc = fmaf(a, a, acc);
        return acc;
    }
};

// ---------------------------------------------------------------------------------
// gradient norms: per-tile sums of squares
// ---------------------------------------------------------------------------------

// grid (n_tiles, K), block 256.  partials[k][tile] = sum over the tile of g[k][i]^2.
// Each lane issues 8 independent 8-byte streaming loads per trip and keeps one fp32
// accumulator per load; with the occupancy capped at 4 waves per SIMD this shape measured
// fastest for a read-only stream on this part (7.3-7.4 TB/s; 16-byte loads at full occupancy
// 6.9-7.0).  An accumulator chain is tile_elems/256/8 elements long (8 for the longest tile);
// everything after the lane is fp64.
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

    float acc[GRAWA_SUMSQ_U];
#pragma unroll
    for (int u = 0; u < GRAWA_SUMSQ_U; ++u) acc[u] = 0.f;

    // unaligned head (< V elements) on the first lanes, tail on the lanes of the second wave
    if (tid < (int)(a_al - a)) {
        const float v = Grad<GT>::one(row + a + tid);
        acc[0] = v * v;
    }
    if (tid >= GRAWA_WAVE && tid - GRAWA_WAVE < (int)(b - b_al)) {
        const float v = Grad<GT>::one(row + b_al + (tid - GRAWA_WAVE));
        acc[1] = v * v;
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
            const float r = Grad<GT>::sumsq8(q[u], 0.f);
            acc[u] += (j0 + u * GRAWA_BLOCK < nvec) ? r : 0.f;
        }
    }

    __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
    double lane = 0.0;
#pragma unroll
    for (int u = 0; u < GRAWA_SUMSQ_U; ++u) lane += (double)acc[u];
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
__device__ __forceinline__ void group_weights(const double *sA, int K, float *beta, int64_t stride,
                                              float *beta_user)
{
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    double mn = INFINITY, nz = 0.0;
    for (int k = lane; k < K; k += GRAWA_WAVE) {
        const double a = sA[k];
        mn = fmin(mn, a);
        nz += (a == 0.0) ? 1.0 : 0.0;
    }
    const double a_min = wave_min(mn);
    const double n_zero = wave_sum(nz);
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
    float *__restrict__ beta, float *__restrict__ beta_user, double *__restrict__ mvg, double gamma)
{
    __shared__ double sA[GRAWA_MAX_WORKERS];
    __shared__ double sw[GRAWA_FIN_WAVES];
    const int l = blockIdx.x;
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
        if (threadIdx.x < K) {
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
    if (wave == 0) group_weights(sA, K, beta + l, L, beta_user ? beta_user + l : nullptr);
}

// Weights from the running norm estimate g_est = scale * g_mvg (Appendix G; scale =
// gamma / (1 - gamma^t)).  per_layer: grid L, block l normalises column l over the workers
// (eq. (7)); otherwise grid 1: score of worker k is the sum of its layer estimates (eq. (3)
// applied to the estimates), then eq. (4).  est_user (float [K][L], may be null) receives g_est.
__global__ __launch_bounds__(GRAWA_FIN_BLOCK) void k_local_weights(const double *__restrict__ mvg, double scale,
                                                                   int K, int L, int per_layer,
                                                                   float *__restrict__ beta,
                                                                   float *__restrict__ beta_user,
                                                                   float *__restrict__ est_user)
{
    __shared__ double sA[GRAWA_MAX_WORKERS];
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    const int wave = threadIdx.x / GRAWA_WAVE;
    if (per_layer) {
        const int l = blockIdx.x;
        for (int k = threadIdx.x; k < K; k += GRAWA_FIN_BLOCK) {
            const double e = scale * mvg[(int64_t)k * L + l];
            sA[k] = e;
            if (est_user) est_user[(int64_t)k * L + l] = (float)e;
        }
        __syncthreads();
        if (wave == 0) group_weights(sA, K, beta + l, L, beta_user ? beta_user + l : nullptr);
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
        if (wave == 0) group_weights(sA, K, beta, 1, beta_user);
    }
}

__global__ __launch_bounds__(GRAWA_BLOCK) void k_zero_f64(double *__restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * GRAWA_BLOCK + threadIdx.x;
    if (i < n) p[i] = 0.0;
}

// grid 1, block 1024.  Model-level score per worker from the [K][L] squared layer norms:
// mode 0: sum of the layer norms; mode 1: norm of the flattened gradient.  Then the K weights.
__global__ __launch_bounds__(GRAWA_FIN_BLOCK) void k_finalize_model(const double *__restrict__ S, int K,
                                                                    int L, int mode,
                                                                    float *__restrict__ beta,
                                                                    float *__restrict__ beta_user)
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
    if (wave == 0) group_weights(sA, K, beta, 1, beta_user);
}

// ---------------------------------------------------------------------------------
// center + pull (+ SGD on the way in)
// ---------------------------------------------------------------------------------

#define GRAWA_CELL 256 // columns per block of the center+pull pass (one per lane)

// Layer of column i, given a layer at or before it (cells that contain a layer boundary).
__device__ __forceinline__ int layer_of(const int64_t *__restrict__ off, int layer, int L, int64_t i)
{
    while (layer + 1 < L && off[layer + 1] <= i) ++layer;
    return layer;
}

// grid ceil(P/256), block 256.  Lane t of block m owns column i = 256 m + t: it loads
// x[k][i] for all K workers (K independent loads in flight; with SGD also g[k][i] and applies
// x - lr g), forms c = sum_k beta_k x_k and writes x_k + lambda (c - x_k) back, so every
// parameter is read once and written once.  A wave touches one 256-byte piece per row.
// KT = number of register slots; EXACT says K == KT (no per-row guards, the usual case),
// otherwise K <= KT.  NT = streaming loads/stores, chosen by the host only when every row
// starts on a 128-byte boundary.  Row bases are wave-uniform, the lane adds only its index.
// cell_layer[m] >= 0: the whole block lies in that layer (weights come through scalar
// loads); < 0: the block contains a layer boundary, ~cell_layer[m] is the layer of its first
// column and each lane finds its own layer.  Model-level weights pass cell_layer = nullptr.
// The pull is x + lambda (c - x), one fma, which leaves a single worker exactly unchanged.
// moving != 0 (EASGD, Appendix F): center_out holds the previous center c0 on entry and the
// center used and stored is c0 + rho (c - c0).
// WPE caps the waves per SIMD: the pass is fastest with roughly 32-48 row loads in flight per
// SIMD (K x WPE); more only queues requests to K far-apart rows and costs DRAM efficiency
// (measured: K = 16 at 3 waves 6.1 TB/s, at 8 waves 5.7; K = 8 at 4 waves 6.5, at 8 waves 6.2).
template <int KT, bool EXACT, bool SGD, typename GT, bool NT, int WPE>
__global__ __launch_bounds__(GRAWA_CELL) __attribute__((amdgpu_waves_per_eu(1, WPE))) void k_center_pull(
    float *__restrict__ x, int64_t ldx, const GT *__restrict__ g, int64_t ldg, float lr,
    const float *__restrict__ beta, int64_t beta_stride, const int32_t *__restrict__ cell_layer,
    const int64_t *__restrict__ off, int L, int K, int64_t P, float lambda,
    float *__restrict__ center_out, float rho, int moving)
{
    const int64_t cell0 = (int64_t)blockIdx.x * GRAWA_CELL; // wave-uniform
    const unsigned t = threadIdx.x;
    const bool ok = cell0 + t < P;
    float *xb = x + cell0;
    const GT *gb = g + cell0;
    const unsigned xoff = t * 4u, goff = t * (unsigned)sizeof(GT);
    const int nk = EXACT ? KT : K;

    float v[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) v[k] = 0.f;
    if (ok) {
#pragma unroll
        for (int k = 0; k < KT; ++k)
            if (k < nk) v[k] = ld_lane<NT, float>(uniform_base(xb + (int64_t)k * ldx), xoff);
        if (SGD) {
#pragma unroll
            for (int k = 0; k < KT; ++k)
                if (k < nk)
                    v[k] = fmaf(-lr, Grad<GT>::template lane<NT>(uniform_base(gb + (int64_t)k * ldg), goff), v[k]);
        }
    }
    float cprev = 0.f;
    if (moving && ok) cprev = ld_lane<NT, float>(uniform_base(center_out + cell0), xoff);

    const int info = cell_layer ? cell_layer[blockIdx.x] : 0;
    float c = 0.f;
    if (info >= 0) { // one layer for the whole block: weights through scalar loads
        const uint64_t bb = uniform_base(beta + info);
#pragma unroll
        for (int k = 0; k < KT; ++k)
            if (k < nk) c = fmaf(ld_uniform_f32(bb, (int64_t)k * beta_stride), v[k], c);
    } else if (ok) { // the block holds a layer boundary: each lane looks up its own layer
        const float *b = beta + layer_of(off, ~info, L, cell0 + t);
#pragma unroll
        for (int k = 0; k < KT; ++k)
            if (k < nk) c = fmaf(b[(int64_t)k * beta_stride], v[k], c);
    }
    if (moving) c = fmaf(rho, c - cprev, cprev);

    if (ok) {
#pragma unroll
        for (int k = 0; k < KT; ++k)
            if (k < nk) st_lane<NT, float>(uniform_base(xb + (int64_t)k * ldx), xoff, fmaf(lambda, c - v[k], v[k]));
        if (center_out) st_lane<NT, float>(uniform_base(center_out + cell0), xoff, c);
    }
}

// Any number of workers: two sweeps over k per column (the second sweep re-reads what the
// first just fetched, normally from cache).  Used only when K exceeds the register-resident
// variants above.
template <bool SGD, typename GT>
__global__ __launch_bounds__(GRAWA_CELL) void k_center_pull_any(
    float *__restrict__ x, int64_t ldx, const GT *__restrict__ g, int64_t ldg, float lr,
    const float *__restrict__ beta, int64_t beta_stride, const int32_t *__restrict__ cell_layer,
    const int64_t *__restrict__ off, int L, int K, int64_t P, float lambda,
    float *__restrict__ center_out, float rho, int moving)
{
    const int64_t i = (int64_t)blockIdx.x * GRAWA_CELL + threadIdx.x;
    if (i >= P) return;
    int layer = 0;
    if (cell_layer) {
        const int info = cell_layer[blockIdx.x];
        layer = info >= 0 ? info : layer_of(off, ~info, L, i);
    }
    const float *b = beta + layer;
    float c = 0.f;
    for (int k = 0; k < K; ++k) {
        float v = x[(int64_t)k * ldx + i];
        if (SGD) v = fmaf(-lr, Grad<GT>::one(g + (int64_t)k * ldg + i), v);
        c = fmaf(b[(int64_t)k * beta_stride], v, c);
    }
    if (moving) c = fmaf(rho, c - center_out[i], center_out[i]);
    for (int k = 0; k < K; ++k) {
        float v = x[(int64_t)k * ldx + i];
        if (SGD) v = fmaf(-lr, Grad<GT>::one(g + (int64_t)k * ldg + i), v);
        x[(int64_t)k * ldx + i] = fmaf(lambda, c - v, v);
    }
    if (center_out) center_out[i] = c;
}

// ---------------------------------------------------------------------------------
// local SGD step
// ---------------------------------------------------------------------------------

// Vector shape of the per-row local steps: a lane handles U vectors of V adjacent columns.  fp32
// gradients: V = 1, U = 4; bf16: V = 2, U = 2 (measured: 6.6-6.7 TB/s for both; bf16 at V = 4, U = 4
// 5.7, at V = 1 4.5; more bytes in flight per lane cost bandwidth at full occupancy).
#define GRAWA_SGD_V_F32 1
#define GRAWA_SGD_U_F32 4
#define GRAWA_SGD_V_BF16 2
#define GRAWA_SGD_U_BF16 2

// V gradient elements (V * sizeof(GT) = 4 or 8 bytes, naturally aligned) widened to float.
template <typename GT, int V, bool NT> struct GradVec;
template <bool NT> struct GradVec<float, 1, NT> {
    static __device__ __forceinline__ void load(const float *p, float (&f)[1]) { f[0] = NT ? __builtin_nontemporal_load(p) : *p; }
};
template <bool NT> struct GradVec<uint16_t, 2, NT> {
    static __device__ __forceinline__ void load(const uint16_t *p, float (&f)[2])
    {
        const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
        const uint32_t w = NT ? __builtin_nontemporal_load(q) : *q;
        f[0] = bf16_lo(w);
        f[1] = bf16_hi(w);
    }
};
template <bool NT> struct GradVec<uint16_t, 4, NT> {
    static __device__ __forceinline__ void load(const uint16_t *p, float (&f)[4])
    {
        const v2u *q = reinterpret_cast<const v2u *>(p);
        const v2u w = NT ? __builtin_nontemporal_load(q) : *q;
        f[0] = bf16_lo(w.x);
        f[1] = bf16_hi(w.x);
        f[2] = bf16_lo(w.y);
        f[3] = bf16_hi(w.y);
    }
};
template <int V> struct FloatVec { typedef float T __attribute__((ext_vector_type(V))); };
template <> struct FloatVec<1> { typedef float T; };
template <int V> __device__ __forceinline__ float vec_get(const typename FloatVec<V>::T &v, int c)
{
    if constexpr (V == 1) return v;
    else return v[c];
}
template <int V> __device__ __forceinline__ void vec_set(typename FloatVec<V>::T &v, int c, float f)
{
    if constexpr (V == 1) v = f;
    else v[c] = f;
}

// grid (ceil(P / (256*U*V)), K), block 256.  x[k][i] -= lr * g[k][i].  A lane handles U vectors of
// V adjacent columns, vectors of a block 256*V columns apart.  Rows start 16-byte aligned, so every
// vector is naturally aligned; the last P % V columns of a row take a scalar path.
template <typename GT, int V, int U, bool NT>
__global__ __launch_bounds__(GRAWA_CELL) void k_local_sgd(float *__restrict__ x, int64_t ldx,
                                                          const GT *__restrict__ g, int64_t ldg,
                                                          int64_t P, float lr)
{
    typedef typename FloatVec<V>::T XV;
    const int64_t nvec = P / V;
    const int64_t j0 = (int64_t)blockIdx.x * (GRAWA_CELL * U) + threadIdx.x;
    float *xr = x + (int64_t)blockIdx.y * ldx;
    const GT *gr = g + (int64_t)blockIdx.y * ldg;
    XV xv[U];
    float gf[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t j = j0 + u * GRAWA_CELL;
        if (j < nvec) {
            const XV *xp = reinterpret_cast<const XV *>(xr + j * V);
            xv[u] = NT ? __builtin_nontemporal_load(xp) : *xp;
            GradVec<GT, V, NT>::load(gr + j * V, gf[u]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t j = j0 + u * GRAWA_CELL;
        if (j < nvec) {
            XV o = xv[u];
#pragma unroll
            for (int c = 0; c < V; ++c) vec_set<V>(o, c, fmaf(-lr, gf[u][c], vec_get<V>(xv[u], c)));
            XV *xp = reinterpret_cast<XV *>(xr + j * V);
            if (NT) __builtin_nontemporal_store(o, xp);
            else *xp = o;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(P - nvec * V)) {
        const int64_t i = nvec * V + threadIdx.x;
        xr[i] = fmaf(-lr, Grad<GT>::one(gr + i), xr[i]);
    }
}

// grid and lane layout of k_local_sgd.  One step of SGD with Nesterov momentum and weight decay
// (the local optimizer of Appendix B.2.2), buf = momentum buffer [K][ldb], zero before the first step:
//     d = g + wd x ;  buf <- momentum buf + d ;  x <- x - lr (d + momentum buf).
template <typename GT, int V, int U, bool NT>
__global__ __launch_bounds__(GRAWA_CELL) void k_nesterov(float *__restrict__ x, int64_t ldx,
                                                         const GT *__restrict__ g, int64_t ldg,
                                                         float *__restrict__ buf, int64_t ldb, int64_t P,
                                                         float lr, float momentum, float wd)
{
    typedef typename FloatVec<V>::T XV;
    const int64_t nvec = P / V;
    const int64_t j0 = (int64_t)blockIdx.x * (GRAWA_CELL * U) + threadIdx.x;
    float *xr = x + (int64_t)blockIdx.y * ldx;
    float *br = buf + (int64_t)blockIdx.y * ldb;
    const GT *gr = g + (int64_t)blockIdx.y * ldg;
    XV xv[U], bv[U];
    float gf[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t j = j0 + u * GRAWA_CELL;
        if (j < nvec) {
            const XV *xp = reinterpret_cast<const XV *>(xr + j * V);
            const XV *bp = reinterpret_cast<const XV *>(br + j * V);
            xv[u] = NT ? __builtin_nontemporal_load(xp) : *xp;
            bv[u] = NT ? __builtin_nontemporal_load(bp) : *bp;
            GradVec<GT, V, NT>::load(gr + j * V, gf[u]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t j = j0 + u * GRAWA_CELL;
        if (j < nvec) {
            XV xo = xv[u], bo = bv[u];
#pragma unroll
            for (int c = 0; c < V; ++c) {
                const float xc = vec_get<V>(xv[u], c);
                const float d = fmaf(wd, xc, gf[u][c]);
                const float b = fmaf(momentum, vec_get<V>(bv[u], c), d);
                vec_set<V>(bo, c, b);
                vec_set<V>(xo, c, fmaf(-lr, fmaf(momentum, b, d), xc));
            }
            XV *xp = reinterpret_cast<XV *>(xr + j * V);
            XV *bp = reinterpret_cast<XV *>(br + j * V);
            if (NT) {
                __builtin_nontemporal_store(xo, xp);
                __builtin_nontemporal_store(bo, bp);
            } else {
                *xp = xo;
                *bp = bo;
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(P - nvec * V)) {
        const int64_t i = nvec * V + threadIdx.x;
        const float xc = xr[i];
        const float d = fmaf(wd, xc, Grad<GT>::one(gr + i));
        const float b = fmaf(momentum, br[i], d);
        br[i] = b;
        xr[i] = fmaf(-lr, fmaf(momentum, b, d), xc);
    }
}

// SGD step of one worker over one aligned block of 1024 columns, with the sums of squares of the
// gradient (for the running norm estimate of Appendix G) taken from the values already in
// registers: grid (ceil(P/1024), K), block 256, V * U * 256 = 1024.  The loads are issued at once;
// only afterwards does the block look at the 1024-column tile map (tiles block_tile0[m] ..
// block_tile0[m+1]-1 lie in aligned block m, each inside one layer) to file its sums:
// partials[k][tile] in fp64.  Nearly every block holds one tile; a block that contains layer
// boundaries reduces once per tile over the columns of that tile.  The last P % V columns of a row
// are handled element by element.  fp32 gradients V = 1, U = 4; bf16 V = 4, U = 1.
template <typename GT, int V, int U, bool NT>
__global__ __launch_bounds__(GRAWA_CELL) void k_row_step_scored(float *__restrict__ x, int64_t ldx,
                                                                const GT *__restrict__ g, int64_t ldg, float lr,
                                                                int64_t P, const GrawaTile *__restrict__ tiles,
                                                                const int32_t *__restrict__ block_tile0,
                                                                int64_t n_tiles, double *__restrict__ partials)
{
    static_assert(V * U * GRAWA_CELL == 1024, "one trip covers one aligned block of the tile map");
    typedef typename FloatVec<V>::T XV;
    __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
    const int64_t c0 = (int64_t)blockIdx.x * 1024 + (int64_t)threadIdx.x * V;
    float *xr = x + (int64_t)blockIdx.y * ldx;
    const GT *gr = g + (int64_t)blockIdx.y * ldg;
    XV xv[U];
    float gf[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = c0 + (int64_t)u * (GRAWA_CELL * V);
        if (c + V <= P) {
            const XV *xp = reinterpret_cast<const XV *>(xr + c);
            xv[u] = NT ? __builtin_nontemporal_load(xp) : *xp;
            GradVec<GT, V, NT>::load(gr + c, gf[u]);
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) gf[u][e] = 0.f;
        }
    }
    const int r0 = block_tile0[blockIdx.x], r1 = block_tile0[blockIdx.x + 1];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = c0 + (int64_t)u * (GRAWA_CELL * V);
        if (c + V <= P) {
            XV o = xv[u];
#pragma unroll
            for (int e = 0; e < V; ++e) vec_set<V>(o, e, fmaf(-lr, gf[u][e], vec_get<V>(xv[u], e)));
            XV *xp = reinterpret_cast<XV *>(xr + c);
            if (NT) __builtin_nontemporal_store(o, xp);
            else *xp = o;
        } else if (V > 1 && c < P) { // the vector that holds the row's last columns
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (c + e < P) {
                    gf[u][e] = Grad<GT>::one(gr + c + e);
                    xr[c + e] = fmaf(-lr, gf[u][e], xr[c + e]);
                }
        }
    }
    double *out = partials + (int64_t)blockIdx.y * n_tiles;
    if (r1 - r0 == 1) { // the usual case: the whole block lies in one tile
        float acc = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int e = 0; e < V; ++e) acc = fmaf(gf[u][e], gf[u][e], acc);
        const double tot = block_sum((double)acc, sm);
        if (threadIdx.x == 0) out[r0] = tot;
    } else {
        for (int r = r0; r < r1; ++r) {
            const int64_t lo = tiles[r].start, hi = lo + tiles[r].len;
            float acc = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const int64_t c = c0 + (int64_t)u * (GRAWA_CELL * V) + e;
                    acc = (c >= lo && c < hi) ? fmaf(gf[u][e], gf[u][e], acc) : acc;
                }
            const double tot = block_sum((double)acc, sm);
            if (threadIdx.x == 0) out[r] = tot;
        }
    }
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

// Local step of all K workers over one tile of columns (Algorithms 1 and 2; Appendix G):
//     x_k <- x_k - lr g_k ;   PROX: x_k <- x_k + w (c - x_k), c a stored center, w = mu/tau ;
//     SCORE: partials[k][tile] = sum over the tile of g_k^2  (for the running norm estimate).
// grid n_tiles, block 256.  The block walks its tile in aligned chunks of 256 columns; per chunk a
// lane owns one column and all K rows of it (2K loads in flight, the stored center read once for
// all K rows), as in the center+pull pass.  tiles == nullptr: uniform tiles of tile_elems columns.
// Tiles are kept short (256 columns without scores, 1024 with): blocks that run together then
// cover one compact window of every row, which measured 10-15 % faster than 4096-16384-column
// tiles (software-pipelining the chunk loop made no difference).
template <int KT, bool EXACT, typename GT, bool NT, bool PROX, bool SCORE, int WPE>
__global__ __launch_bounds__(GRAWA_CELL) __attribute__((amdgpu_waves_per_eu(1, WPE))) void k_rows_step(
    float *__restrict__ x, int64_t ldx, const GT *__restrict__ g, int64_t ldg, float lr,
    const float *__restrict__ center, float w, const GrawaTile *__restrict__ tiles, int tile_elems,
    int64_t n_tiles, int K, int64_t P, double *__restrict__ partials)
{
    int64_t a, b;
    if (tiles) {
        const GrawaTile tl = tiles[blockIdx.x];
        a = tl.start;
        b = tl.start + tl.len;
    } else {
        a = (int64_t)blockIdx.x * tile_elems;
        b = a + tile_elems < P ? a + tile_elems : P;
    }
    const unsigned t = threadIdx.x;
    const int nk = EXACT ? KT : K;
    float acc[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) acc[k] = 0.f;

    for (int64_t c0 = a - (a % GRAWA_CELL); c0 < b; c0 += GRAWA_CELL) { // c0 is wave-uniform
        const int64_t i = c0 + t;
        const bool ok = i >= a && i < b;
        const unsigned xoff = t * 4u, goff = t * (unsigned)sizeof(GT);
        float v[KT], gv[KT];
        float cv = 0.f;
        if (ok) {
#pragma unroll
            for (int k = 0; k < KT; ++k)
                if (k < nk) v[k] = ld_lane<NT, float>(uniform_base(x + (int64_t)k * ldx + c0), xoff);
#pragma unroll
            for (int k = 0; k < KT; ++k)
                if (k < nk) gv[k] = Grad<GT>::template lane<NT>(uniform_base(g + (int64_t)k * ldg + c0), goff);
            if (PROX) cv = ld_lane<false, float>(uniform_base(center + c0), xoff);
            __builtin_amdgcn_sched_barrier(0); // every load of the chunk is issued before the first is used
#pragma unroll
            for (int k = 0; k < KT; ++k)
                if (k < nk) {
                    float r = fmaf(-lr, gv[k], v[k]);
                    if (PROX) r = fmaf(w, cv - r, r);
                    if (SCORE) acc[k] = fmaf(gv[k], gv[k], acc[k]);
                    st_lane<NT, float>(uniform_base(x + (int64_t)k * ldx + c0), xoff, r);
                }
        }
    }

    if (SCORE) {
        __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
        for (int k = 0; k < nk; ++k) {
            float ak = 0.f;
#pragma unroll
            for (int kk = 0; kk < KT; ++kk) ak = (kk == k) ? acc[kk] : ak; // keeps acc[] in registers
            const double tot = block_sum((double)ak, sm);
            if (t == 0) partials[(int64_t)k * n_tiles + blockIdx.x] = tot;
        }
    }
}

// ---------------------------------------------------------------------------------
// plain copy (measurement aid)
// ---------------------------------------------------------------------------------

// grid ceil(n/64), block 64 (one wave): one streaming 16-byte load and store per lane, the
// shape that measured fastest for a two-stream copy on this part.
#define GRAWA_COPY_BLOCK 64
__global__ __launch_bounds__(GRAWA_COPY_BLOCK) void k_stream_copy(v4u *__restrict__ dst,
                                                                  const v4u *__restrict__ src, int64_t n)
{
    const int64_t j = (int64_t)blockIdx.x * GRAWA_COPY_BLOCK + threadIdx.x;
    if (j < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + j), dst + j);
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
        p->d_beta_layer, beta_user, update_estimate ? p->d_mvg : nullptr, gamma);
    return hipGetLastError();
}

hipError_t grawa_launch_local_weights(const grawa_plan *p, double scale, int per_layer, float *beta_user,
                                      float *est_user, hipStream_t s)
{
    k_local_weights<<<dim3(per_layer ? (unsigned)p->L : 1u), dim3(GRAWA_FIN_BLOCK), 0, s>>>(
        p->d_mvg, scale, p->K, p->L, per_layer, per_layer ? p->d_beta_layer : p->d_beta_model, beta_user,
        est_user);
    return hipGetLastError();
}

hipError_t grawa_launch_zero_estimate(const grawa_plan *p, hipStream_t s)
{
    const int64_t n = (int64_t)p->K * p->L;
    k_zero_f64<<<dim3((unsigned)((n + GRAWA_BLOCK - 1) / GRAWA_BLOCK)), dim3(GRAWA_BLOCK), 0, s>>>(p->d_mvg, n);
    return hipGetLastError();
}

hipError_t grawa_launch_finalize_model(const grawa_plan *p, grawa_norm_mode_t mode, float *beta_user,
                                       hipStream_t s)
{
    k_finalize_model<<<dim3(1), dim3(GRAWA_FIN_BLOCK), 0, s>>>(p->d_S, p->K, p->L, (int)mode,
                                                          p->d_beta_model, beta_user);
    return hipGetLastError();
}

// Waves per SIMD the center+pull kernel is capped at, from a sweep of this kernel over K and
// the cap on the part (best throughput at roughly 32-48 row loads in flight per SIMD).
constexpr int grawa_waves_for(int k, bool sgd)
{
    if (sgd) return k <= 2 ? 8 : k == 3 ? 6 : k <= 5 ? 5 : k <= 7 ? 4 : k <= 11 ? 3 : 2;
    return k <= 4 ? 8 : k == 5 ? 6 : k <= 7 ? 5 : k <= 10 ? 4 : k <= 20 ? 3 : k <= 28 ? 2 : 1;
}

template <int KT, bool EXACT, bool SGD, typename GT, bool NT>
static void launch_cp(const grawa_plan *p, float *x, int64_t ldx, const void *g, int64_t ldg, float lr,
                      const float *beta, int per_layer, float lambda, float *center_out, float rho, int moving,
                      hipStream_t s, hipEvent_t e0, hipEvent_t e1)
{
    hipExtLaunchKernelGGL((k_center_pull<KT, EXACT, SGD, GT, NT, grawa_waves_for(KT, SGD)>),
                          dim3((unsigned)p->n_cells), dim3(GRAWA_CELL), 0, s, e0, e1, 0, x, ldx, (const GT *)g, ldg,
                          lr, beta, per_layer ? (int64_t)p->L : (int64_t)1,
                          per_layer ? (const int32_t *)p->d_cell_layer : (const int32_t *)nullptr,
                          (const int64_t *)p->d_off, p->L, p->K, p->P, lambda, center_out, rho, moving);
}

// One kernel per worker count up to 32 (fully unrolled, no guards); 33..64 workers share a
// guarded 64-slot kernel; beyond that the two-sweep kernel.
template <bool SGD, typename GT, bool NT>
static void dispatch_cp(const grawa_plan *p, float *x, int64_t ldx, const void *g, int64_t ldg, float lr,
                        const float *beta, int per_layer, float lambda, float *center_out, float rho, int moving,
                        hipStream_t s, hipEvent_t e0, hipEvent_t e1)
{
#define GRAWA_CP_CASE(N) \
    case N: launch_cp<N, true, SGD, GT, NT>(p, x, ldx, g, ldg, lr, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1); break;
    const int K = p->K;
    switch (K) {
        GRAWA_CP_CASE(1) GRAWA_CP_CASE(2) GRAWA_CP_CASE(3) GRAWA_CP_CASE(4) GRAWA_CP_CASE(5) GRAWA_CP_CASE(6)
        GRAWA_CP_CASE(7) GRAWA_CP_CASE(8) GRAWA_CP_CASE(9) GRAWA_CP_CASE(10) GRAWA_CP_CASE(11) GRAWA_CP_CASE(12)
        GRAWA_CP_CASE(13) GRAWA_CP_CASE(14) GRAWA_CP_CASE(15) GRAWA_CP_CASE(16) GRAWA_CP_CASE(17) GRAWA_CP_CASE(18)
        GRAWA_CP_CASE(19) GRAWA_CP_CASE(20) GRAWA_CP_CASE(21) GRAWA_CP_CASE(22) GRAWA_CP_CASE(23) GRAWA_CP_CASE(24)
        GRAWA_CP_CASE(25) GRAWA_CP_CASE(26) GRAWA_CP_CASE(27) GRAWA_CP_CASE(28) GRAWA_CP_CASE(29) GRAWA_CP_CASE(30)
        GRAWA_CP_CASE(31) GRAWA_CP_CASE(32)
    default:
        if (K <= 64)
            launch_cp<64, false, SGD, GT, NT>(p, x, ldx, g, ldg, lr, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1);
        else
            hipExtLaunchKernelGGL((k_center_pull_any<SGD, GT>), dim3((unsigned)p->n_cells), dim3(GRAWA_CELL), 0, s,
                                  e0, e1, 0, x, ldx, (const GT *)g, ldg, lr, beta,
                                  per_layer ? (int64_t)p->L : (int64_t)1,
                                  per_layer ? (const int32_t *)p->d_cell_layer : (const int32_t *)nullptr,
                                  (const int64_t *)p->d_off, p->L, K, p->P, lambda, center_out, rho, moving);
    }
#undef GRAWA_CP_CASE
}

#define GRAWA_STREAMING_MIN_BYTES ((int64_t)512 << 20)

// Streaming accesses are used only when no cache line is shared between two rows or written
// in two parts: base pointers and row pitches are multiples of 128 bytes.
static bool rows_line_aligned(const void *base, int64_t ld, int elem_bytes)
{
    return (reinterpret_cast<uintptr_t>(base) % 128u) == 0 && ((ld * elem_bytes) % 128) == 0;
}

hipError_t grawa_launch_center_pull(const grawa_plan *p, float *x, int64_t ldx, const float *beta,
                                    int per_layer, float lambda, const void *g_sgd, int64_t ldg_sgd,
                                    grawa_dtype_t dt, float lr, int fuse_sgd, float *center_out, float rho,
                                    int moving, hipStream_t s, hipEvent_t e0, hipEvent_t e1)
{
    // Streaming accesses pay off only when the arrays do not fit the last-level cache anyway.
    bool nt = (int64_t)p->K * p->P * 4 > GRAWA_STREAMING_MIN_BYTES && rows_line_aligned(x, ldx, 4) &&
              (!center_out || rows_line_aligned(center_out, 0, 4));
    if (fuse_sgd) nt = nt && rows_line_aligned(g_sgd, ldg_sgd, dt == GRAWA_BF16 ? 2 : 4);
    if (!fuse_sgd) {
        if (nt) dispatch_cp<false, float, true>(p, x, ldx, nullptr, 0, 0.f, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1);
        else dispatch_cp<false, float, false>(p, x, ldx, nullptr, 0, 0.f, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1);
    } else if (dt == GRAWA_BF16) {
        if (nt) dispatch_cp<true, uint16_t, true>(p, x, ldx, g_sgd, ldg_sgd, lr, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1);
        else dispatch_cp<true, uint16_t, false>(p, x, ldx, g_sgd, ldg_sgd, lr, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1);
    } else {
        if (nt) dispatch_cp<true, float, true>(p, x, ldx, g_sgd, ldg_sgd, lr, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1);
        else dispatch_cp<true, float, false>(p, x, ldx, g_sgd, ldg_sgd, lr, beta, per_layer, lambda, center_out, rho, moving, s, e0, e1);
    }
    return hipGetLastError();
}

hipError_t grawa_launch_local_sgd(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt,
                                  int K, int64_t P, float lr, hipStream_t s)
{
    const int64_t per_block = dt == GRAWA_BF16 ? GRAWA_CELL * GRAWA_SGD_U_BF16 * GRAWA_SGD_V_BF16
                                               : GRAWA_CELL * GRAWA_SGD_U_F32 * GRAWA_SGD_V_F32;
    int64_t gx = (P + per_block - 1) / per_block;
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, (unsigned)K), block(GRAWA_CELL);
    const bool nt = (int64_t)K * P * 4 > GRAWA_STREAMING_MIN_BYTES && rows_line_aligned(x, ldx, 4) &&
                    rows_line_aligned(g, ldg, dt == GRAWA_BF16 ? 2 : 4);
#define GRAWA_SGD_GO(GT, V, U, NT) k_local_sgd<GT, V, U, NT><<<grid, block, 0, s>>>(x, ldx, (const GT *)g, ldg, P, lr)
    if (dt == GRAWA_BF16) {
        if (nt) GRAWA_SGD_GO(uint16_t, GRAWA_SGD_V_BF16, GRAWA_SGD_U_BF16, true);
        else GRAWA_SGD_GO(uint16_t, GRAWA_SGD_V_BF16, GRAWA_SGD_U_BF16, false);
    } else {
        if (nt) GRAWA_SGD_GO(float, GRAWA_SGD_V_F32, GRAWA_SGD_U_F32, true);
        else GRAWA_SGD_GO(float, GRAWA_SGD_V_F32, GRAWA_SGD_U_F32, false);
    }
#undef GRAWA_SGD_GO
    return hipGetLastError();
}

hipError_t grawa_launch_nesterov(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt, float *buf,
                                 int64_t ldb, int K, int64_t P, float lr, float momentum, float wd, hipStream_t s)
{
    const int64_t per_block = dt == GRAWA_BF16 ? GRAWA_CELL * GRAWA_SGD_U_BF16 * GRAWA_SGD_V_BF16
                                               : GRAWA_CELL * GRAWA_SGD_U_F32 * GRAWA_SGD_V_F32;
    int64_t gx = (P + per_block - 1) / per_block;
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, (unsigned)K), block(GRAWA_CELL);
    const bool nt = (int64_t)K * P * 4 > GRAWA_STREAMING_MIN_BYTES && rows_line_aligned(x, ldx, 4) &&
                    rows_line_aligned(buf, ldb, 4) && rows_line_aligned(g, ldg, dt == GRAWA_BF16 ? 2 : 4);
#define GRAWA_NAG_GO(GT, V, U, NT) \
    k_nesterov<GT, V, U, NT><<<grid, block, 0, s>>>(x, ldx, (const GT *)g, ldg, buf, ldb, P, lr, momentum, wd)
    if (dt == GRAWA_BF16) {
        if (nt) GRAWA_NAG_GO(uint16_t, GRAWA_SGD_V_BF16, GRAWA_SGD_U_BF16, true);
        else GRAWA_NAG_GO(uint16_t, GRAWA_SGD_V_BF16, GRAWA_SGD_U_BF16, false);
    } else {
        if (nt) GRAWA_NAG_GO(float, GRAWA_SGD_V_F32, GRAWA_SGD_U_F32, true);
        else GRAWA_NAG_GO(float, GRAWA_SGD_V_F32, GRAWA_SGD_U_F32, false);
    }
#undef GRAWA_NAG_GO
    return hipGetLastError();
}

// Per-row scored step; tiles / block_tile0: the plan's 1024-column tile map and its index by aligned block.
hipError_t grawa_launch_row_step_scored(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt,
                                        float lr, const GrawaTile *tiles, const int32_t *block_tile0,
                                        int64_t n_tiles, int K, int64_t P, double *partials, hipStream_t s)
{
    const dim3 grid((unsigned)((P + 1023) / 1024), (unsigned)K), block(GRAWA_CELL);
    const bool nt = (int64_t)K * P * 4 > GRAWA_STREAMING_MIN_BYTES && rows_line_aligned(x, ldx, 4) &&
                    rows_line_aligned(g, ldg, dt == GRAWA_BF16 ? 2 : 4);
#define GRAWA_RSS_GO(GT, V, U, NT)                                                                             \
    k_row_step_scored<GT, V, U, NT><<<grid, block, 0, s>>>(x, ldx, (const GT *)g, ldg, lr, P, tiles, block_tile0, \
                                                           n_tiles, partials)
    if (dt == GRAWA_BF16) {
        if (nt) GRAWA_RSS_GO(uint16_t, 4, 1, true);
        else GRAWA_RSS_GO(uint16_t, 4, 1, false);
    } else {
        if (nt) GRAWA_RSS_GO(float, 1, 4, true);
        else GRAWA_RSS_GO(float, 1, 4, false);
    }
#undef GRAWA_RSS_GO
    return hipGetLastError();
}

hipError_t grawa_launch_center_weights(const grawa_plan *p, const float *loss, float *beta_user, int *leader_out,
                                       hipStream_t s)
{
    k_center_weights<<<dim3(1), dim3(GRAWA_WAVE), 0, s>>>(loss, p->K, p->d_beta_model, beta_user, leader_out);
    return hipGetLastError();
}

// K-row local step: SGD (+ proximity step) (+ per-tile sums of squares of the gradient).
template <int KT, bool EXACT, typename GT, bool NT, bool PROX, bool SCORE>
static void launch_rows(float *x, int64_t ldx, const void *g, int64_t ldg, float lr, const float *center, float w,
                        const GrawaTile *tiles, int tile_elems, int64_t n_tiles, int K, int64_t P,
                        double *partials, hipStream_t s)
{
    k_rows_step<KT, EXACT, GT, NT, PROX, SCORE, grawa_waves_for(KT, true)>
        <<<dim3((unsigned)n_tiles), dim3(GRAWA_CELL), 0, s>>>(x, ldx, (const GT *)g, ldg, lr, center, w, tiles,
                                                             tile_elems, n_tiles, K, P, partials);
}

template <typename GT, bool NT, bool PROX, bool SCORE>
static bool dispatch_rows(float *x, int64_t ldx, const void *g, int64_t ldg, float lr, const float *center, float w,
                          const GrawaTile *tiles, int tile_elems, int64_t n_tiles, int K, int64_t P,
                          double *partials, hipStream_t s)
{
#define GRAWA_ROWS_CASE(N) \
    case N: launch_rows<N, true, GT, NT, PROX, SCORE>(x, ldx, g, ldg, lr, center, w, tiles, tile_elems, n_tiles, K, P, partials, s); break;
    switch (K) {
        GRAWA_ROWS_CASE(1) GRAWA_ROWS_CASE(2) GRAWA_ROWS_CASE(3) GRAWA_ROWS_CASE(4) GRAWA_ROWS_CASE(5) GRAWA_ROWS_CASE(6)
        GRAWA_ROWS_CASE(7) GRAWA_ROWS_CASE(8) GRAWA_ROWS_CASE(9) GRAWA_ROWS_CASE(10) GRAWA_ROWS_CASE(11) GRAWA_ROWS_CASE(12)
        GRAWA_ROWS_CASE(13) GRAWA_ROWS_CASE(14) GRAWA_ROWS_CASE(15) GRAWA_ROWS_CASE(16) GRAWA_ROWS_CASE(24)
        GRAWA_ROWS_CASE(32)
    default:
        if (K > 64) return false;
        if (K <= 32) launch_rows<32, false, GT, NT, PROX, SCORE>(x, ldx, g, ldg, lr, center, w, tiles, tile_elems, n_tiles, K, P, partials, s);
        else launch_rows<64, false, GT, NT, PROX, SCORE>(x, ldx, g, ldg, lr, center, w, tiles, tile_elems, n_tiles, K, P, partials, s);
    }
#undef GRAWA_ROWS_CASE
    return true;
}

// Returns hipErrorInvalidValue when K exceeds what the kernel family covers (K > 64).
hipError_t grawa_launch_rows_step(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt, float lr,
                                  const float *center, float w, const GrawaTile *tiles, int tile_elems,
                                  int64_t n_tiles, int K, int64_t P, double *partials, hipStream_t s)
{
    const bool nt = (int64_t)K * P * 4 > GRAWA_STREAMING_MIN_BYTES && rows_line_aligned(x, ldx, 4) &&
                    rows_line_aligned(g, ldg, dt == GRAWA_BF16 ? 2 : 4);
    const bool prox = center != nullptr, score = partials != nullptr;
    bool ok;
#define GRAWA_ROWS_GO(GT, NT, PROX, SCORE) \
    ok = dispatch_rows<GT, NT, PROX, SCORE>(x, ldx, g, ldg, lr, center, w, tiles, tile_elems, n_tiles, K, P, partials, s)
#define GRAWA_ROWS_PS(GT, NT)                         \
    do {                                              \
        if (prox && score) GRAWA_ROWS_GO(GT, NT, true, true);   \
        else if (prox) GRAWA_ROWS_GO(GT, NT, true, false);      \
        else if (score) GRAWA_ROWS_GO(GT, NT, false, true);     \
        else GRAWA_ROWS_GO(GT, NT, false, false);               \
    } while (0)
    if (dt == GRAWA_BF16) {
        if (nt) GRAWA_ROWS_PS(uint16_t, true);
        else GRAWA_ROWS_PS(uint16_t, false);
    } else {
        if (nt) GRAWA_ROWS_PS(float, true);
        else GRAWA_ROWS_PS(float, false);
    }
#undef GRAWA_ROWS_PS
#undef GRAWA_ROWS_GO
    if (!ok) return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t grawa_launch_stream_copy(void *dst, const void *src, int64_t nbytes, hipStream_t s)
{
    const int64_t n = nbytes / 16;
    const int64_t gx = (n + GRAWA_COPY_BLOCK - 1) / GRAWA_COPY_BLOCK;
    if (gx > 0)
        k_stream_copy<<<dim3((unsigned)gx), dim3(GRAWA_COPY_BLOCK), 0, s>>>((v4u *)dst, (const v4u *)src, n);
    return hipGetLastError();
}
