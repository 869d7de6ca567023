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

// grid ceil(P/C), block S*C.  Thread t of block m owns column i = C m + (t mod C) and the rows of
// row group t / C: it loads x[k][i] for its KT/S workers (all loads in flight together; with SGD
// also g[k][i] and applies x - lr g), forms its part of c = sum_k beta_k x_k, the S parts are added
// through LDS, and it writes x_k + lambda (c - x_k) back, so every parameter is read once and written
// once.  A wave touches one 256-byte piece per row.  S = 1, C = 256 is the plain form (one lane owns a
// whole column, no LDS, no barrier).
// KT = number of register slots per column; EXACT says K == KT (no per-row guards, the usual case),
// otherwise K <= KT (S = 1 only).  NT = streaming loads/stores, chosen by the host only when every row
// starts on a 128-byte boundary.  Row bases are wave-uniform, the lane adds only its index.
// cell_layer[j] describes the 256-column cell j: >= 0: the whole cell lies in that layer (weights
// come through scalar loads); < 0: the cell contains a layer boundary, ~cell_layer[j] is the layer of
// its first column and each lane finds its own layer.  Model-level weights pass cell_layer = nullptr.
// The pull is x + lambda (c - x), one fma, which leaves a single worker exactly unchanged.
// moving != 0 (EASGD, Appendix F): center_out holds the previous center c0 on entry and the
// center used and stored is c0 + rho (c - c0).
// WPE caps the waves per SIMD: the plain form is fastest with roughly 32-48 row loads in flight per
// SIMD (K x WPE); more only queues requests to K far-apart rows and costs DRAM efficiency
// (measured: K = 16 at 3 waves 6.1 TB/s, at 8 waves 5.7; K = 8 at 4 waves 6.5, at 8 waves 6.2).
// Splitting the rows over S groups of waves (4 rows per wave, the whole block starting its loads
// and, after the barrier, its stores together) measured 1-2 % faster than the plain form for 16
// workers; for every other worker count tried (6 to 32, with and without the SGD step) the plain
// form at its best occupancy cap is as fast or faster on arrays of random values.
template <int KT, bool EXACT, bool SGD, typename GT, bool NT, int WPE, int S, int C>
__global__ __launch_bounds__(S *C) __attribute__((amdgpu_waves_per_eu(1, WPE))) void k_center_pull(
    float *__restrict__ x, int64_t ldx, const GT *__restrict__ g, int64_t ldg, float lr,
    const float *__restrict__ beta, int64_t beta_stride, const int32_t *__restrict__ cell_layer,
    const int64_t *__restrict__ off, int L, int K, int64_t P, float lambda,
    float *__restrict__ center_out, float rho, int moving)
{
    static_assert(S == 1 || (EXACT && KT % S == 0), "row groups need an exact, evenly divided worker count");
    static_assert(C % GRAWA_WAVE == 0 && GRAWA_CELL % C == 0, "a block covers whole waves inside one cell");
    constexpr int KS = KT / S; // rows per thread
    const int64_t cell0 = (int64_t)blockIdx.x * C; // wave-uniform
    const unsigned col = S == 1 ? threadIdx.x : threadIdx.x % C;
    const int k0 = S == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x / C) * KS); // wave-uniform
    const bool ok = cell0 + col < P;
    float *xb = x + cell0 + (int64_t)k0 * ldx;
    const GT *gb = g + cell0 + (int64_t)k0 * ldg;
    const unsigned xoff = col * 4u, goff = col * (unsigned)sizeof(GT);
    const int nk = EXACT ? KS : K;

    float v[KS];
#pragma unroll
    for (int k = 0; k < KS; ++k) v[k] = 0.f;
    if (ok) {
#pragma unroll
        for (int k = 0; k < KS; ++k)
            if (k < nk) v[k] = ld_lane<NT, float>(uniform_base(xb + (int64_t)k * ldx), xoff);
        if (SGD) {
#pragma unroll
            for (int k = 0; k < KS; ++k)
                if (k < nk)
                    v[k] = fmaf(-lr, Grad<GT>::template lane<NT>(uniform_base(gb + (int64_t)k * ldg), goff), v[k]);
        }
    }
    float cprev = 0.f;
    if (moving && ok) cprev = ld_lane<NT, float>(uniform_base(center_out + cell0), xoff);

    const int info = cell_layer ? cell_layer[cell0 / GRAWA_CELL] : 0;
    float c = 0.f;
    if (info >= 0) { // one layer for the whole cell: weights through scalar loads
        const uint64_t bb = uniform_base(beta + info + (int64_t)k0 * beta_stride);
#pragma unroll
        for (int k = 0; k < KS; ++k)
            if (k < nk) c = fmaf(ld_uniform_f32(bb, (int64_t)k * beta_stride), v[k], c);
    } else if (ok) { // the cell holds a layer boundary: each lane looks up its own layer
        const float *b = beta + layer_of(off, ~info, L, cell0 + col) + (int64_t)k0 * beta_stride;
#pragma unroll
        for (int k = 0; k < KS; ++k)
            if (k < nk) c = fmaf(b[(int64_t)k * beta_stride], v[k], c);
    }
    if (S > 1) { // add the row groups' parts, in group order
        __shared__ float part[S][C];
        part[threadIdx.x / C][col] = c;
        __syncthreads();
        c = 0.f;
#pragma unroll
        for (int s = 0; s < S; ++s) c += part[s][col];
    }
    if (moving) c = fmaf(rho, c - cprev, cprev);

    if (ok) {
#pragma unroll
        for (int k = 0; k < KS; ++k)
            if (k < nk) st_lane<NT, float>(uniform_base(xb + (int64_t)k * ldx), xoff, fmaf(lambda, c - v[k], v[k]));
        if (center_out && k0 == 0) st_lane<NT, float>(uniform_base(center_out + cell0), xoff, c);
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

// Waves per SIMD the center+pull kernel is capped at, from sweeps of this kernel over K and
// the cap on the part, on arrays of 3 to 11 GB holding random values (best throughput at roughly
// 24-48 row loads in flight per SIMD).  The values matter: arrays of zeros stream about 4 % faster
// on this part and shift some of the optima, so sweeps over cleared memory mislead.
constexpr int grawa_waves_for(int k, bool sgd)
{
    if (sgd) return k <= 3 ? 8 : k <= 5 ? 5 : k <= 7 ? 4 : k <= 11 ? 3 : 2;
    return k <= 4 ? 8 : k == 5 ? 5 : k <= 8 ? 4 : k <= 16 ? 3 : k <= 28 ? 2 : 1;
}

// Row groups S and columns per block C by worker count: the plain form except where the split form
// measured faster on arrays of random values (16 workers without the SGD step).
template <int KT, bool SGD> struct CpShape { static constexpr int S = 1, C = GRAWA_CELL; };
template <> struct CpShape<16, false> { static constexpr int S = 4, C = 256; };

template <int KT, bool EXACT, bool SGD, typename GT, bool NT>
static void launch_cp(const grawa_plan *p, float *x, int64_t ldx, const void *g, int64_t ldg, float lr,
                      const float *beta, int per_layer, float lambda, float *center_out, float rho, int moving,
                      hipStream_t s, hipEvent_t e0, hipEvent_t e1)
{
    constexpr int S = EXACT ? CpShape<KT, SGD>::S : 1, C = EXACT ? CpShape<KT, SGD>::C : GRAWA_CELL;
    constexpr int WPE = S == 1 ? grawa_waves_for(KT, SGD) : 8;
    const unsigned grid = (unsigned)((p->P + C - 1) / C);
    hipExtLaunchKernelGGL((k_center_pull<KT, EXACT, SGD, GT, NT, WPE, S, C>), dim3(grid), dim3(S * C), 0, s, e0, e1, 0,
                          x, ldx, (const GT *)g, ldg, lr, beta, per_layer ? (int64_t)p->L : (int64_t)1,
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
