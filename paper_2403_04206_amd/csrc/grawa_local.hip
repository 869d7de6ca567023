// Local-phase kernels of the GRAWA training loop (gfx950, wave64):
//   k_row_step     x_k <- x_k - lr g_k                                            [Alg. 1, 2]
//                  (+ proximity step toward the stored center)                    [Alg. 1, 2, "Prox."]
//                  (+ per-tile sums of squares of the gradient, for the running
//                     norm estimate of Local-GRAWA)                               [App. G]
//   k_nesterov     SGD with Nesterov momentum and weight decay                   [App. B.2.2]
//   k_stream_copy  plain copy (measurement aid)
// All are read-modify-write streams with no reuse: global loads and stores kept in flight, one
// row (worker) per block, which is the access shape that streams fastest on this part.
#include "grawa_device.h"

// ---------------------------------------------------------------------------------
// local step, row by row
// ---------------------------------------------------------------------------------

#define GRAWA_ROW_BLOCK 1024 // columns per block
#define GRAWA_ROW_GROUP 4096 // column blocks of one row launched back to back (4 Mi columns)

// One block = one aligned block of 1024 columns of one worker; V * U * 256 = 1024, a lane handles U
// vectors of V adjacent columns.  All loads are issued at once, then
//     x <- x - lr g ;   PROX: x <- x + w (c - x), c the stored center, w = mu/tau ;
//     SCORE: partials[k][tile] = sum over the tile of g^2 in fp64, from the values in registers.
// grid (group, K, n_groups): the column blocks are cut into groups of gridDim.x; blocks are started
// with x fastest, so within a group the blocks of worker 0 come first, then worker 1, ..., and no
// index arithmetic is needed to find a block's place.  Blocks that run together therefore stream one
// row (the fastest shape: 6.4-6.6 TB/s against 5.2-6.0 for a block that owns all K rows of a
// tile), and the piece of the center a group needs (16 MB) is re-read by the other K-1 workers
// from cache instead of HBM.  With one group per row pass (k slowest) the center is re-read from
// HBM once it outgrows the last-level cache (measured 4.5 TB/s at P = 354 M); with k fastest the
// blocks in flight spread over all K rows (5.8-6.0).
// SCORE: only after its loads are issued does a block consult the 1024-column tile map (tiles
// block_tile0[m] .. block_tile0[m+1]-1 lie in aligned block m, each inside one layer).  Nearly
// every block holds one tile; a block that contains layer boundaries reduces once per tile.
// The last P % V columns of a row are handled element by element.
template <typename GT, int V, int U, bool NT, bool PROX, bool SCORE>
__global__ __launch_bounds__(GRAWA_CELL) void k_row_step(float *__restrict__ x, int64_t ldx,
                                                         const GT *__restrict__ g, int64_t ldg, float lr,
                                                         const float *__restrict__ center, float w, int64_t P,
                                                         unsigned n_blocks,
                                                         const GrawaTile *__restrict__ tiles,
                                                         const int32_t *__restrict__ block_tile0, int64_t n_tiles,
                                                         double *__restrict__ partials)
{
    static_assert(V * U * GRAWA_CELL == GRAWA_ROW_BLOCK, "one trip covers one aligned block of columns");
    typedef typename FloatVec<V>::T XV;
    __shared__ double sm[GRAWA_BLOCK / GRAWA_WAVE];
    const unsigned k = blockIdx.y;
    const unsigned m = blockIdx.z * gridDim.x + blockIdx.x;
    if (m >= n_blocks) return; // the last group may be short (whole block leaves, before any barrier)
    const int64_t c0 = (int64_t)m * GRAWA_ROW_BLOCK + (int64_t)threadIdx.x * V;
    float *xr = x + (int64_t)k * ldx;
    const GT *gr = g + (int64_t)k * ldg;
    XV xv[U], cv[U];
    float gf[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = c0 + (int64_t)u * (GRAWA_CELL * V);
        if (c + V <= P) {
            const XV *xp = reinterpret_cast<const XV *>(xr + c);
            xv[u] = NT ? __builtin_nontemporal_load(xp) : *xp;
            GradVec<GT, V, NT>::load(gr + c, gf[u]);
            if (PROX) cv[u] = *reinterpret_cast<const XV *>(center + c); // cached: shared by the K rows
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) gf[u][e] = 0.f;
        }
    }
    int r0 = 0, r1 = 1;
    if (SCORE) {
        r0 = block_tile0[m];
        r1 = block_tile0[m + 1];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t c = c0 + (int64_t)u * (GRAWA_CELL * V);
        if (c + V <= P) {
            XV o = xv[u];
#pragma unroll
            for (int e = 0; e < V; ++e) {
                float v = fmaf(-lr, gf[u][e], vec_get<V>(xv[u], e));
                if (PROX) v = fmaf(w, vec_get<V>(cv[u], e) - v, v);
                vec_set<V>(o, e, v);
            }
            XV *xp = reinterpret_cast<XV *>(xr + c);
            if (NT) __builtin_nontemporal_store(o, xp);
            else *xp = o;
        } else if (V > 1 && c < P) { // the vector that holds the row's last columns
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (c + e < P) {
                    gf[u][e] = Grad<GT>::one(gr + c + e);
                    float v = fmaf(-lr, gf[u][e], xr[c + e]);
                    if (PROX) v = fmaf(w, center[c + e] - v, v);
                    xr[c + e] = v;
                }
        }
    }
    if (!SCORE) return;
    double *out = partials + (int64_t)k * n_tiles;
    if (r1 - r0 == 1) { // the usual case: the whole block lies in one tile
        double acc = 0.0; // squares and sums in fp64: exact squares at any gradient magnitude
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int e = 0; e < V; ++e) acc = sq_add(gf[u][e], acc);
        const double tot = block_sum(acc, sm);
        if (threadIdx.x == 0) out[r0] = tot;
    } else {
        for (int t = r0; t < r1; ++t) {
            const int64_t lo = tiles[t].start, hi = lo + tiles[t].len;
            double acc = 0.0;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const int64_t c = c0 + (int64_t)u * (GRAWA_CELL * V) + e;
                    acc = (c >= lo && c < hi) ? sq_add(gf[u][e], acc) : acc;
                }
            const double tot = block_sum(acc, sm);
            if (threadIdx.x == 0) out[t] = tot;
        }
    }
}

// ---------------------------------------------------------------------------------
// Nesterov-momentum SGD step
// ---------------------------------------------------------------------------------

// Vector shape of the Nesterov step: fp32 gradients V = 1, U = 4; bf16 V = 2, U = 2 (measured
// 6.3-6.4 TB/s for both; bf16 at V = 4, U = 4 5.6: more bytes in flight per lane cost bandwidth at
// full occupancy, and 2-byte loads (V = 1) waste requests).
#define GRAWA_SGD_V_F32 1
#define GRAWA_SGD_U_F32 4
#define GRAWA_SGD_V_BF16 2
#define GRAWA_SGD_U_BF16 2

// grid (ceil(P / (256*U*V)), K), block 256; a lane handles U vectors of V adjacent columns, vectors of a
// block 256*V columns apart; the last P % V columns of a row take a scalar path.  One step of SGD with Nesterov momentum and weight decay
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

// center == nullptr: no proximity step.  partials == nullptr: no scores (tiles, block_tile0 and
// n_tiles are then unused); otherwise they are the plan's 1024-column tile map, its index by
// aligned block and its length.  Vector shapes: fp32 gradients V = 1, U = 4 for the plain step,
// V = 4, U = 1 with the proximity step or the scores; bf16 V = 2, U = 2 for the plain step, else
// V = 4, U = 1 (each the fastest measured for its case on arrays of random values; the spread
// between shapes is 3-10 %).
hipError_t grawa_launch_row_step(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt, float lr,
                                 const float *center, float w, int K, int64_t P, const GrawaTile *tiles,
                                 const int32_t *block_tile0, int64_t n_tiles, double *partials, hipStream_t s)
{
    const int64_t nb = (P + GRAWA_ROW_BLOCK - 1) / GRAWA_ROW_BLOCK;
    const bool prox = center != nullptr, score = partials != nullptr;
    // Nothing is shared between the rows without a center: one group, i.e. row after row (3 % faster).
    const int64_t group = (prox && nb > GRAWA_ROW_GROUP) ? GRAWA_ROW_GROUP : nb;
    const int64_t n_groups = (nb + group - 1) / group;
    if (K > 65535 || n_groups > 65535 || group >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)group, (unsigned)K, (unsigned)n_groups), block(GRAWA_CELL);
    const bool nt = (int64_t)K * P * 4 > GRAWA_STREAMING_MIN_BYTES && rows_line_aligned(x, ldx, 4) &&
                    rows_line_aligned(g, ldg, dt == GRAWA_BF16 ? 2 : 4);
#define GRAWA_RS_GO(GT, V, U, NT, PROX, SCORE)                                                                   \
    k_row_step<GT, V, U, NT, PROX, SCORE><<<grid, block, 0, s>>>(x, ldx, (const GT *)g, ldg, lr, center, w, P, \
                                                                 (unsigned)nb, tiles, block_tile0, n_tiles,    \
                                                                 partials)
#define GRAWA_RS_NT(GT, V, U, PROX, SCORE)              \
    do {                                                \
        if (nt) GRAWA_RS_GO(GT, V, U, true, PROX, SCORE); \
        else GRAWA_RS_GO(GT, V, U, false, PROX, SCORE);   \
    } while (0)
    if (dt == GRAWA_BF16) {
        if (prox && score) GRAWA_RS_NT(uint16_t, 4, 1, true, true);
        else if (prox) GRAWA_RS_NT(uint16_t, 4, 1, true, false);
        else if (score) GRAWA_RS_NT(uint16_t, 4, 1, false, true);
        else GRAWA_RS_NT(uint16_t, 2, 2, false, false);
    } else {
        if (prox && score) GRAWA_RS_NT(float, 4, 1, true, true);
        else if (prox) GRAWA_RS_NT(float, 4, 1, true, false);
        else if (score) GRAWA_RS_NT(float, 4, 1, false, true);
        else GRAWA_RS_NT(float, 1, 4, false, false);
    }
#undef GRAWA_RS_NT
#undef GRAWA_RS_GO
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

hipError_t grawa_launch_stream_copy(void *dst, const void *src, int64_t nbytes, hipStream_t s)
{
    const int64_t n = nbytes / 16;
    const int64_t gx = (n + GRAWA_COPY_BLOCK - 1) / GRAWA_COPY_BLOCK;
    if (gx > 0)
        k_stream_copy<<<dim3((unsigned)gx), dim3(GRAWA_COPY_BLOCK), 0, s>>>((v4u *)dst, (const v4u *)src, n);
    return hipGetLastError();
}
