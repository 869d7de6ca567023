// Local-phase kernels of the GRAWA training loop (gfx950, wave64):
//   k_local_sgd        x_k <- x_k - lr g_k                                       [Alg. 1, 2]
//   k_nesterov         SGD with Nesterov momentum and weight decay               [App. B.2.2]
//   k_row_step_scored  SGD step + per-tile gradient sums of squares              [App. G]
//   k_rows_step        SGD step + proximity step toward the stored center
//                      (+ per-tile gradient sums of squares)                     [Alg. 1, 2; App. G]
//   k_stream_copy      plain copy (measurement aid)
// All are read-modify-write streams with no reuse: global loads and stores kept in flight.
#include "grawa_device.h"

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
