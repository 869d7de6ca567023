// Center and pull of the GRAWA update (gfx950, wave64):
//   x_C = sum_k beta_k x_k ;  x_k <- x_k + lambda (x_C - x_k)      [display after eq. (2); eq. (7)]
// with the local SGD step x_k - lr g_k optionally applied on the way in (Algorithms 1 and 2) and,
// for EASGD (Appendix F), the center averaged in time.
//
// A read-modify-write pass over K far-apart rows: it runs fastest when a wave touches one aligned
// 256-byte piece of every row (one 32-bit element per lane per row), blocks are small and many,
// and accesses are non-temporal -- provided every row starts on a 128-byte boundary, so that no
// cache line is written in two parts.  There is no dense contraction, hence no matrix-core code.
#include "grawa_device.h"

// ---------------------------------------------------------------------------------
// center + pull (+ SGD on the way in)
// ---------------------------------------------------------------------------------

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
// launchers
// ---------------------------------------------------------------------------------

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
