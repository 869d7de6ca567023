// HIP kernels of the GRAWA distributed update for gfx950 (MI355X), wave64.
//
// The update is a streaming computation: every parameter and gradient element is read
// once per pass and there is no reuse, so each kernel is built around 128-bit global
// loads/stores, many of them in flight per lane, and nothing else.  There is no dense
// contraction here and therefore no matrix-core code.
//
//   k_sumsq            per (tile, worker) sum of squares of the gradient   [eq. (3), (5)]
//   k_finalize_layers  per layer: tile partials -> ||G||_F^2, ||G||_F, per-layer weights
//                                                                          [eq. (5)-(7)]
//   k_finalize_model   per worker: model score, model-level weights        [eq. (2)-(4)]
//   k_center_pull      x_C = sum_k beta_k x_k ; x_k <- x_k + lambda (x_C - x_k), with the
//                      local SGD step x_k - lr g_k optionally applied on the way in
//                                                   [display after eq. (2); Alg. 1, 2]
//   k_local_sgd        x_k <- x_k - lr g_k                                 [Alg. 1, 2]
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

// Sum / min over the block through LDS; every thread gets the result.  `sm` holds one
// double per wave.  Safe to call repeatedly with the same `sm`.
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

__device__ __forceinline__ double block_min(double v, double *sm)
{
    v = wave_min(v);
    const int w = threadIdx.x / GRAWA_WAVE;
    __syncthreads();
    if ((threadIdx.x & (GRAWA_WAVE - 1)) == 0) sm[w] = v;
    __syncthreads();
    double t = sm[0];
    for (int i = 1; i < GRAWA_BLOCK / GRAWA_WAVE; ++i) t = fmin(t, sm[i]);
    return t;
}

// Gradient element access.  VEC16 = elements per 16-byte load (norm pass); a "quad" is 4
// consecutive elements (what one lane handles next to one float4 of parameters).
template <typename GT> struct Grad;

template <> struct Grad<float> {
    static constexpr int VEC16 = 4;
    static __device__ __forceinline__ float one(const float *p) { return *p; }
    static __device__ __forceinline__ float sumsq16(const float *p, float acc)
    {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        acc = fmaf(q.x, q.x, acc);
        acc = fmaf(q.y, q.y, acc);
        acc = fmaf(q.z, q.z, acc);
        acc = fmaf(q.w, q.w, acc);
        return acc;
    }
    static __device__ __forceinline__ float4 quad(const float *p) { return *reinterpret_cast<const float4 *>(p); }
};

template <> struct Grad<uint16_t> { // bfloat16 bit patterns
    static constexpr int VEC16 = 8;
    static __device__ __forceinline__ float one(const uint16_t *p) { return bf16_one(*p); }
    static __device__ __forceinline__ float sumsq16(const uint16_t *p, float acc)
    {
        const uint4 q = *reinterpret_cast<const uint4 *>(p);
        float a;
        a = bf16_lo(q.x); acc = fmaf(a, a, acc);
        a = bf16_hi(q.x); acc = fmaf(a, a, acc);
        a = bf16_lo(q.y); acc = fmaf(a, a, acc);
        a = bf16_hi(q.y); acc = fmaf(a, a, acc);
        a = bf16_lo(q.z); acc = fmaf(a, a, acc);
        a = bf16_hi(q.z); acc = fmaf(a, a, acc);
        a = bf16_lo(q.w); acc = fmaf(a, a, acc);
        a = bf16_hi(q.w); acc = fmaf(a, a, acc);
        return acc;
    }
    static __device__ __forceinline__ float4 quad(const uint16_t *p)
    {
        const uint2 q = *reinterpret_cast<const uint2 *>(p);
        return make_float4(bf16_lo(q.x), bf16_hi(q.x), bf16_lo(q.y), bf16_hi(q.y));
    }
};

// ---------------------------------------------------------------------------------
// gradient norms: per-tile sums of squares
// ---------------------------------------------------------------------------------

// grid (n_tiles, K), block 256.  partials[k][tile] = sum over the tile of g[k][i]^2.
// Each lane keeps 4 independent fp32 accumulators (one per load of an unrolled group of
// four 16-byte loads), so a chain is at most tile_elems/256/4 elements long; everything
// after the lane is fp64.
template <typename GT>
__global__ __launch_bounds__(GRAWA_BLOCK) void k_sumsq(const GT *__restrict__ g, int64_t ldg,
                                                       const GrawaTile *__restrict__ tiles,
                                                       int64_t n_tiles,
                                                       double *__restrict__ partials)
{
    constexpr int V = Grad<GT>::VEC16;
    const GrawaTile t = tiles[blockIdx.x];
    const int k = blockIdx.y;
    const GT *row = g + (int64_t)k * ldg;
    const int tid = threadIdx.x;

    const int64_t a = t.start, b = t.start + t.len;
    int64_t a_al = (a + V - 1) / V * V;
    if (a_al > b) a_al = b;
    int64_t b_al = b / V * V;
    if (b_al < a_al) b_al = a_al;

    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;

    // unaligned head (< V elements) on the first lanes, tail on the lanes of the second wave
    if (tid < (int)(a_al - a)) {
        const float v = Grad<GT>::one(row + a + tid);
        acc0 = v * v;
    }
    if (tid >= GRAWA_WAVE && tid - GRAWA_WAVE < (int)(b - b_al)) {
        const float v = Grad<GT>::one(row + b_al + (tid - GRAWA_WAVE));
        acc1 = v * v;
    }

    const int nvec = (int)((b_al - a_al) / V);
    const GT *body = row + a_al;
    int j = tid;
    for (; j + 3 * GRAWA_BLOCK < nvec; j += 4 * GRAWA_BLOCK) {
        acc0 = Grad<GT>::sumsq16(body + (int64_t)j * V, acc0);
        acc1 = Grad<GT>::sumsq16(body + (int64_t)(j + GRAWA_BLOCK) * V, acc1);
        acc2 = Grad<GT>::sumsq16(body + (int64_t)(j + 2 * GRAWA_BLOCK) * V, acc2);
        acc3 = Grad<GT>::sumsq16(body + (int64_t)(j + 3 * GRAWA_BLOCK) * V, acc3);
    }
    if (j < nvec) acc0 = Grad<GT>::sumsq16(body + (int64_t)j * V, acc0);
    if (j + GRAWA_BLOCK < nvec) acc1 = Grad<GT>::sumsq16(body + (int64_t)(j + GRAWA_BLOCK) * V, acc1);
    if (j + 2 * GRAWA_BLOCK < nvec) acc2 = Grad<GT>::sumsq16(body + (int64_t)(j + 2 * GRAWA_BLOCK) * V, acc2);

    __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
    const double lane = ((double)acc0 + (double)acc1) + ((double)acc2 + (double)acc3);
    const double total = block_sum(lane, sm);
    if (tid == 0) partials[(int64_t)k * n_tiles + blockIdx.x] = total;
}

// ---------------------------------------------------------------------------------
// weights
// ---------------------------------------------------------------------------------

// Weights of one group of K scores held in LDS (sA[k], k < K): beta_k proportional to
// 1/A_k, summing to one, evaluated as (A_min/A_k) / sum_j (A_min/A_j) so that nothing
// overflows.  Scores of exactly zero share the weight equally and take all of it (the
// limit A -> 0+).  Every thread of the block must call this.
__device__ __forceinline__ void group_weights(const double *sA, int K, float *beta, int64_t stride,
                                              float *beta_user, double *sm)
{
    double mn = INFINITY, nz = 0.0;
    for (int k = threadIdx.x; k < K; k += GRAWA_BLOCK) {
        const double a = sA[k];
        mn = fmin(mn, a);
        nz += (a == 0.0) ? 1.0 : 0.0;
    }
    const double a_min = block_min(mn, sm);
    const double n_zero = block_sum(nz, sm);
    double z = 0.0;
    if (n_zero == 0.0)
        for (int k = threadIdx.x; k < K; k += GRAWA_BLOCK) z += a_min / sA[k];
    const double zsum = block_sum(z, sm);
    for (int k = threadIdx.x; k < K; k += GRAWA_BLOCK) {
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

// grid L, block 256.  Block l adds the tile partials of layer l for every worker (one wave
// per worker at a time, lanes striding over the layer's tiles), then turns the K layer
// norms into the K per-layer weights.
__global__ __launch_bounds__(GRAWA_BLOCK) void k_finalize_layers(
    const double *__restrict__ partials, int64_t n_tiles, const int32_t *__restrict__ layer_tile0,
    int K, int L, double *__restrict__ S, float *__restrict__ A, float *__restrict__ A_user,
    float *__restrict__ beta, float *__restrict__ beta_user)
{
    __shared__ double sA[GRAWA_MAX_WORKERS];
    __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
    const int l = blockIdx.x;
    const int t0 = layer_tile0[l], t1 = layer_tile0[l + 1];
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    const int wave = threadIdx.x / GRAWA_WAVE;
    for (int k = wave; k < K; k += GRAWA_BLOCK / GRAWA_WAVE) {
        const double *p = partials + (int64_t)k * n_tiles;
        double s = 0.0;
        for (int t = t0 + lane; t < t1; t += GRAWA_WAVE) s += p[t];
        s = wave_sum(s);
        if (lane == 0) {
            const double a = sqrt(s);
            S[(int64_t)k * L + l] = s;
            A[(int64_t)k * L + l] = (float)a;
            if (A_user) A_user[(int64_t)k * L + l] = (float)a;
            sA[k] = a;
        }
    }
    __syncthreads();
    group_weights(sA, K, beta + l, L, beta_user ? beta_user + l : nullptr, sm);
}

// grid 1, block 256.  Model-level score per worker from the [K][L] squared layer norms:
// mode 0: sum of the layer norms; mode 1: norm of the flattened gradient.  Then the K weights.
__global__ __launch_bounds__(GRAWA_BLOCK) void k_finalize_model(const double *__restrict__ S, int K,
                                                                int L, int mode,
                                                                float *__restrict__ beta,
                                                                float *__restrict__ beta_user)
{
    __shared__ double sA[GRAWA_MAX_WORKERS];
    __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
    const int lane = threadIdx.x & (GRAWA_WAVE - 1);
    const int wave = threadIdx.x / GRAWA_WAVE;
    for (int k = wave; k < K; k += GRAWA_BLOCK / GRAWA_WAVE) {
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
    group_weights(sA, K, beta, 1, beta_user, sm);
}

// ---------------------------------------------------------------------------------
// center + pull (+ SGD on the way in)
// ---------------------------------------------------------------------------------

__device__ __forceinline__ float4 axpy4(float a, float4 g, float4 x)
{ // x - a*g, one fma per component
    return make_float4(fmaf(-a, g.x, x.x), fmaf(-a, g.y, x.y), fmaf(-a, g.z, x.z), fmaf(-a, g.w, x.w));
}

// grid n_tiles, block 256.  KT = compile-time bound on the number of workers (K <= KT),
// U = float4 columns a lane handles per trip.  A lane loads its column of all K workers
// into registers (K*U independent 16-byte loads in flight), forms the weighted sum, and
// writes the K pulled values back: every parameter is read once and written once.
// The pull is x + lambda (c - x), one fma, which leaves a single worker exactly unchanged.
template <int KT, int U, bool SGD, typename GT>
__global__ __launch_bounds__(GRAWA_BLOCK) void k_center_pull(
    float *__restrict__ x, int64_t ldx, const GT *__restrict__ g, int64_t ldg, float lr,
    const float *__restrict__ beta, int64_t beta_stride, int per_layer,
    const GrawaTile *__restrict__ tiles, int K, float lambda, float *__restrict__ center_out)
{
    const GrawaTile t = tiles[blockIdx.x];
    const int tid = threadIdx.x;
    const int bcol = per_layer ? t.layer : 0;

    float bk[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) bk[k] = (k < K) ? beta[(int64_t)k * beta_stride + bcol] : 0.f;

    const int64_t a = t.start, b = t.start + t.len;
    int64_t a_al = (a + 3) / 4 * 4;
    if (a_al > b) a_al = b;
    int64_t b_al = b / 4 * 4;
    if (b_al < a_al) b_al = a_al;

    // elements before / after the 16-byte aligned body: one lane each, two sweeps over k
    {
        int64_t i = -1;
        if (tid < (int)(a_al - a)) i = a + tid;
        else if (tid >= GRAWA_WAVE && tid - GRAWA_WAVE < (int)(b - b_al)) i = b_al + (tid - GRAWA_WAVE);
        if (i >= 0) {
            float c = 0.f;
            for (int k = 0; k < K; ++k) {
                float v = x[(int64_t)k * ldx + i];
                if (SGD) v = fmaf(-lr, Grad<GT>::one(g + (int64_t)k * ldg + i), v);
                c = fmaf(beta[(int64_t)k * beta_stride + bcol], v, c);
            }
            for (int k = 0; k < K; ++k) {
                float v = x[(int64_t)k * ldx + i];
                if (SGD) v = fmaf(-lr, Grad<GT>::one(g + (int64_t)k * ldg + i), v);
                x[(int64_t)k * ldx + i] = fmaf(lambda, c - v, v);
            }
            if (center_out) center_out[i] = c;
        }
    }

    const int nvec = (int)((b_al - a_al) / 4);
    float *xb = x + a_al;
    const GT *gb = g + a_al;
    for (int j0 = tid; j0 < nvec; j0 += U * GRAWA_BLOCK) {
        float4 v[U][KT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * GRAWA_BLOCK;
            if (j < nvec) {
#pragma unroll
                for (int k = 0; k < KT; ++k)
                    if (k < K) v[u][k] = *reinterpret_cast<const float4 *>(xb + (int64_t)k * ldx + 4 * (int64_t)j);
                if (SGD) {
#pragma unroll
                    for (int k = 0; k < KT; ++k)
                        if (k < K) v[u][k] = axpy4(lr, Grad<GT>::quad(gb + (int64_t)k * ldg + 4 * (int64_t)j), v[u][k]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * GRAWA_BLOCK;
            if (j < nvec) {
                float4 c = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int k = 0; k < KT; ++k)
                    if (k < K) {
                        c.x = fmaf(bk[k], v[u][k].x, c.x);
                        c.y = fmaf(bk[k], v[u][k].y, c.y);
                        c.z = fmaf(bk[k], v[u][k].z, c.z);
                        c.w = fmaf(bk[k], v[u][k].w, c.w);
                    }
#pragma unroll
                for (int k = 0; k < KT; ++k)
                    if (k < K) {
                        float4 o;
                        o.x = fmaf(lambda, c.x - v[u][k].x, v[u][k].x);
                        o.y = fmaf(lambda, c.y - v[u][k].y, v[u][k].y);
                        o.z = fmaf(lambda, c.z - v[u][k].z, v[u][k].z);
                        o.w = fmaf(lambda, c.w - v[u][k].w, v[u][k].w);
                        *reinterpret_cast<float4 *>(xb + (int64_t)k * ldx + 4 * (int64_t)j) = o;
                    }
                if (center_out) *reinterpret_cast<float4 *>(center_out + a_al + 4 * (int64_t)j) = c;
            }
        }
    }
}

// Any number of workers: two sweeps over k per column (the second sweep re-reads what the
// first just fetched, normally from cache).  Used only when K exceeds the register-resident
// variants above.
template <bool SGD, typename GT>
__global__ __launch_bounds__(GRAWA_BLOCK) void k_center_pull_any(
    float *__restrict__ x, int64_t ldx, const GT *__restrict__ g, int64_t ldg, float lr,
    const float *__restrict__ beta, int64_t beta_stride, int per_layer,
    const GrawaTile *__restrict__ tiles, int K, float lambda, float *__restrict__ center_out)
{
    const GrawaTile t = tiles[blockIdx.x];
    const int bcol = per_layer ? t.layer : 0;
    for (int64_t i = t.start + threadIdx.x; i < t.start + t.len; i += GRAWA_BLOCK) {
        float c = 0.f;
        for (int k = 0; k < K; ++k) {
            float v = x[(int64_t)k * ldx + i];
            if (SGD) v = fmaf(-lr, Grad<GT>::one(g + (int64_t)k * ldg + i), v);
            c = fmaf(beta[(int64_t)k * beta_stride + bcol], v, c);
        }
        for (int k = 0; k < K; ++k) {
            float v = x[(int64_t)k * ldx + i];
            if (SGD) v = fmaf(-lr, Grad<GT>::one(g + (int64_t)k * ldg + i), v);
            x[(int64_t)k * ldx + i] = fmaf(lambda, c - v, v);
        }
        if (center_out) center_out[i] = c;
    }
}

// ---------------------------------------------------------------------------------
// local SGD step
// ---------------------------------------------------------------------------------

#define GRAWA_SGD_U 4 // float4 columns per lane

// grid (ceil(P / (256*4*U)), K), block 256.  x[k][i] -= lr * g[k][i].
template <typename GT>
__global__ __launch_bounds__(GRAWA_BLOCK) void k_local_sgd(float *__restrict__ x, int64_t ldx,
                                                           const GT *__restrict__ g, int64_t ldg,
                                                           int64_t P, float lr)
{
    const int k = blockIdx.y;
    float *xr = x + (int64_t)k * ldx;
    const GT *gr = g + (int64_t)k * ldg;
    const int64_t nvec = P / 4;
    const int64_t j0 = (int64_t)blockIdx.x * (GRAWA_SGD_U * GRAWA_BLOCK) + threadIdx.x;
    float4 xv[GRAWA_SGD_U], gv[GRAWA_SGD_U];
#pragma unroll
    for (int u = 0; u < GRAWA_SGD_U; ++u) {
        const int64_t j = j0 + u * GRAWA_BLOCK;
        if (j < nvec) {
            xv[u] = *reinterpret_cast<const float4 *>(xr + 4 * j);
            gv[u] = Grad<GT>::quad(gr + 4 * j);
        }
    }
#pragma unroll
    for (int u = 0; u < GRAWA_SGD_U; ++u) {
        const int64_t j = j0 + u * GRAWA_BLOCK;
        if (j < nvec) *reinterpret_cast<float4 *>(xr + 4 * j) = axpy4(lr, gv[u], xv[u]);
    }
    // the last P % 4 elements of the row
    if (blockIdx.x == 0 && threadIdx.x < (int)(P - nvec * 4)) {
        const int64_t i = nvec * 4 + threadIdx.x;
        xr[i] = fmaf(-lr, Grad<GT>::one(gr + i), xr[i]);
    }
}

// ---------------------------------------------------------------------------------
// plain copy (measurement aid)
// ---------------------------------------------------------------------------------

__global__ __launch_bounds__(GRAWA_BLOCK) void k_stream_copy(uint4 *__restrict__ dst,
                                                             const uint4 *__restrict__ src, int64_t n)
{
    const int64_t j0 = (int64_t)blockIdx.x * (8 * GRAWA_BLOCK) + threadIdx.x;
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
        if (j0 + u * GRAWA_BLOCK < n) v[u] = src[j0 + u * GRAWA_BLOCK];
#pragma unroll
    for (int u = 0; u < 8; ++u)
        if (j0 + u * GRAWA_BLOCK < n) dst[j0 + u * GRAWA_BLOCK] = v[u];
}

// ---------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------

hipError_t grawa_launch_sumsq(const grawa_plan *p, const void *g, int64_t ldg, grawa_dtype_t dt,
                              hipStream_t s)
{
    const dim3 grid((unsigned)p->n_tiles, (unsigned)p->K), block(GRAWA_BLOCK);
    if (dt == GRAWA_BF16)
        k_sumsq<uint16_t><<<grid, block, 0, s>>>((const uint16_t *)g, ldg, p->d_tiles, p->n_tiles, p->d_partials);
    else
        k_sumsq<float><<<grid, block, 0, s>>>((const float *)g, ldg, p->d_tiles, p->n_tiles, p->d_partials);
    return hipGetLastError();
}

hipError_t grawa_launch_finalize_layers(const grawa_plan *p, float *norms_user, float *beta_user,
                                        hipStream_t s)
{
    k_finalize_layers<<<dim3((unsigned)p->L), dim3(GRAWA_BLOCK), 0, s>>>(
        p->d_partials, p->n_tiles, p->d_layer_tile0, p->K, p->L, p->d_S, p->d_A, norms_user,
        p->d_beta_layer, beta_user);
    return hipGetLastError();
}

hipError_t grawa_launch_finalize_model(const grawa_plan *p, grawa_norm_mode_t mode, float *beta_user,
                                       hipStream_t s)
{
    k_finalize_model<<<dim3(1), dim3(GRAWA_BLOCK), 0, s>>>(p->d_S, p->K, p->L, (int)mode,
                                                          p->d_beta_model, beta_user);
    return hipGetLastError();
}

template <int KT, int U, bool SGD, typename GT>
static void launch_cp(const grawa_plan *p, float *x, int64_t ldx, const void *g, int64_t ldg, float lr,
                      const float *beta, int per_layer, float lambda, float *center_out, hipStream_t s)
{
    k_center_pull<KT, U, SGD, GT><<<dim3((unsigned)p->n_tiles), dim3(GRAWA_BLOCK), 0, s>>>(
        x, ldx, (const GT *)g, ldg, lr, beta, per_layer ? (int64_t)p->L : 1, per_layer, p->d_tiles,
        p->K, lambda, center_out);
}

template <bool SGD, typename GT>
static void dispatch_cp(const grawa_plan *p, float *x, int64_t ldx, const void *g, int64_t ldg, float lr,
                        const float *beta, int per_layer, float lambda, float *center_out, hipStream_t s)
{
    const int K = p->K;
    if (K <= 2) launch_cp<2, 8, SGD, GT>(p, x, ldx, g, ldg, lr, beta, per_layer, lambda, center_out, s);
    else if (K <= 4) launch_cp<4, 4, SGD, GT>(p, x, ldx, g, ldg, lr, beta, per_layer, lambda, center_out, s);
    else if (K <= 8) launch_cp<8, 2, SGD, GT>(p, x, ldx, g, ldg, lr, beta, per_layer, lambda, center_out, s);
    else if (K <= 16) launch_cp<16, 1, SGD, GT>(p, x, ldx, g, ldg, lr, beta, per_layer, lambda, center_out, s);
    else if (K <= 32) launch_cp<32, 1, SGD, GT>(p, x, ldx, g, ldg, lr, beta, per_layer, lambda, center_out, s);
    else
        k_center_pull_any<SGD, GT><<<dim3((unsigned)p->n_tiles), dim3(GRAWA_BLOCK), 0, s>>>(
            x, ldx, (const GT *)g, ldg, lr, beta, per_layer ? (int64_t)p->L : 1, per_layer, p->d_tiles, K,
            lambda, center_out);
}

hipError_t grawa_launch_center_pull(const grawa_plan *p, float *x, int64_t ldx, const float *beta,
                                    int per_layer, float lambda, const void *g_sgd, int64_t ldg_sgd,
                                    grawa_dtype_t dt, float lr, int fuse_sgd, float *center_out,
                                    hipStream_t s)
{
    if (!fuse_sgd)
        dispatch_cp<false, float>(p, x, ldx, nullptr, 0, 0.f, beta, per_layer, lambda, center_out, s);
    else if (dt == GRAWA_BF16)
        dispatch_cp<true, uint16_t>(p, x, ldx, g_sgd, ldg_sgd, lr, beta, per_layer, lambda, center_out, s);
    else
        dispatch_cp<true, float>(p, x, ldx, g_sgd, ldg_sgd, lr, beta, per_layer, lambda, center_out, s);
    return hipGetLastError();
}

hipError_t grawa_launch_local_sgd(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt,
                                  int K, int64_t P, float lr, hipStream_t s)
{
    const int64_t nvec = P / 4;
    int64_t gx = (nvec + GRAWA_SGD_U * GRAWA_BLOCK - 1) / (GRAWA_SGD_U * GRAWA_BLOCK);
    if (gx < 1) gx = 1;
    const dim3 grid((unsigned)gx, (unsigned)K), block(GRAWA_BLOCK);
    if (dt == GRAWA_BF16)
        k_local_sgd<uint16_t><<<grid, block, 0, s>>>(x, ldx, (const uint16_t *)g, ldg, P, lr);
    else
        k_local_sgd<float><<<grid, block, 0, s>>>(x, ldx, (const float *)g, ldg, P, lr);
    return hipGetLastError();
}

hipError_t grawa_launch_stream_copy(void *dst, const void *src, int64_t nbytes, hipStream_t s)
{
    const int64_t n = nbytes / 16;
    const int64_t gx = (n + 8 * GRAWA_BLOCK - 1) / (8 * GRAWA_BLOCK);
    if (gx > 0)
        k_stream_copy<<<dim3((unsigned)gx), dim3(GRAWA_BLOCK), 0, s>>>((uint4 *)dst, (const uint4 *)src, n);
    return hipGetLastError();
}
