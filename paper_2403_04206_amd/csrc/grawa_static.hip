// LGRAWA update for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): the same kernels as grawa_lgrawa_update,
// with the plan's workspace replaced by a fixed array that lives in the library's device image.
// The index maps a plan builds on the host are built here by two small kernels from layer
// offsets that already sit in device memory, so the call enqueues kernels and nothing else.
#include <cstring>
#include <mutex>

#include "grawa_device.h"

#define GRAWA_STATIC_SCRATCH_BYTES ((size_t)32 << 20)

// One copy per GPU the library runs on, held until the process ends.  In host code this name
// is only a handle for the symbol lookup below; the device address comes from that lookup.
static __device__ __align__(256) unsigned char scratch[GRAWA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices]; // device address of `scratch` on every device, looked up once

hipError_t scratch_of_current_device(int *dev_out, void **ptr_out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *dev_out = dev;
    *ptr_out = g_scratch_ptr[dev];
    return hipSuccess;
}

inline size_t round256(size_t n) { return (n + 255) & ~size_t(255); }

} // namespace

// Offsets are read from device memory the host never sees, so they cannot be validated before
// the launch; they are clamped to [0, P] (and made monotone) wherever an address is formed from
// them, which keeps every access in range whatever they hold.
__device__ __forceinline__ int64_t clamp_off(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

#define GRAWA_SCAN_BLOCK 1024

// grid 1, block 1024.  layer_tile0[l] = number of norm-pass tiles before layer l when every layer
// is cut at the multiples of T (the same cut the host-side plan makes); layer_tile0[L] = total.
// Nothing exceeds `bound`, the tile count the host sized the partials for.
__global__ __launch_bounds__(GRAWA_SCAN_BLOCK) void k_static_layer_tiles(const int64_t *__restrict__ off, int L,
                                                                          int64_t P, int T, int64_t bound,
                                                                          int32_t *__restrict__ layer_tile0)
{
    __shared__ int64_t sm[GRAWA_SCAN_BLOCK];
    __shared__ int64_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < L; base += GRAWA_SCAN_BLOCK) {
        const int l = base + tid;
        int64_t cnt = 0;
        if (l < L) {
            const int64_t a = clamp_off(off[l], 0, P), b = clamp_off(off[l + 1], a, P);
            if (b > a) cnt = (b - 1) / T - a / T + 1;
        }
        sm[tid] = cnt;
        __syncthreads();
        for (int d = 1; d < GRAWA_SCAN_BLOCK; d <<= 1) { // inclusive scan
            const int64_t v = tid >= d ? sm[tid - d] : 0;
            __syncthreads();
            sm[tid] += v;
            __syncthreads();
        }
        const int64_t before = carry + sm[tid] - cnt;
        if (l < L) layer_tile0[l] = (int32_t)(before < bound ? before : bound);
        __syncthreads();
        if (tid == GRAWA_SCAN_BLOCK - 1) carry += sm[tid];
        __syncthreads();
    }
    if (tid == 0) layer_tile0[L] = (int32_t)(carry < bound ? carry : bound);
}

// Largest l in [0, L-1] with key[l] <= v (key[0] <= v assumed; key non-decreasing).
template <typename T> __device__ __forceinline__ int last_not_above(const T *__restrict__ key, int L, int64_t v)
{
    int lo = 0, hi = L - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)key[mid] <= v) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// grid ceil(max(bound, n_cells)/256), block 256.  Thread i writes tile i of the norm pass (tiles
// past the real total get length 0: their blocks add nothing) and the layer of 256-column cell i
// of the center+pull pass (the layer itself if the cell lies in one layer, else the complement of
// the layer of its first column).
__global__ __launch_bounds__(GRAWA_BLOCK) void k_static_maps(const int64_t *__restrict__ off, int L, int64_t P, int T,
                                                             int64_t bound, const int32_t *__restrict__ layer_tile0,
                                                             GrawaTile *__restrict__ tiles, int64_t n_cells,
                                                             int32_t *__restrict__ cell_layer)
{
    const int64_t i = (int64_t)blockIdx.x * GRAWA_BLOCK + threadIdx.x;
    if (i < bound) {
        GrawaTile t = {0, 0, 0};
        if (i < layer_tile0[L]) {
            const int l = last_not_above(layer_tile0, L, i);
            const int64_t a = clamp_off(off[l], 0, P), b = clamp_off(off[l + 1], a, P);
            const int64_t j = a / T + (i - layer_tile0[l]);
            int64_t start = j * T, stop = (j + 1) * T;
            if (start < a) start = a;
            if (stop > b) stop = b;
            if (stop < start) stop = start;
            t.start = start;
            t.len = (int32_t)(stop - start);
            t.layer = l;
        }
        tiles[i] = t;
    }
    if (i < n_cells) {
        const int64_t first = i * GRAWA_CELL;
        const int64_t last = (first + GRAWA_CELL < P ? first + GRAWA_CELL : P) - 1;
        const int l = last_not_above(off, L, first);
        cell_layer[i] = off[l + 1] > last ? (int32_t)l : ~(int32_t)l;
    }
}

extern "C" grawa_status_t grawa_lgrawa_update_static(int K, int64_t P, int L, const int64_t *layer_offsets_dev,
                                                     float *x, int64_t ldx, const void *g, int64_t ldg,
                                                     grawa_dtype_t dt, float lambda, float *center_out,
                                                     float *weights_out, void *stream)
{
    if (K < 1 || P < 1 || L < 1 || (int64_t)L > P || !layer_offsets_dev) return GRAWA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(layer_offsets_dev) & 7u) != 0) return GRAWA_ERR_ALIGNMENT;
    if (K > GRAWA_MAX_WORKERS) return GRAWA_ERR_UNSUPPORTED;
    grawa_status_t st;
    if ((st = grawa_check_params(P, x, ldx)) != GRAWA_OK) return st;
    if ((st = grawa_check_grads(P, g, ldg, dt)) != GRAWA_OK) return st;
    if ((st = grawa_check_lambda(lambda)) != GRAWA_OK) return st;
    if ((st = grawa_check_center(center_out)) != GRAWA_OK) return st;

    // The same tile length a plan would choose, so both paths add the same partial sums in the
    // same order.  Tiles: at most one per started multiple of T plus one per layer.
    const int T = grawa_default_tile_elems(K, P);
    const int64_t bound = P / T + L + 1;
    const int64_t nc = (P + GRAWA_CELL - 1) / GRAWA_CELL;
    if (bound > GRAWA_MAX_TILES || nc >= GRAWA_MAX_TILES) return GRAWA_ERR_UNSUPPORTED;
    const size_t b_cells = round256(sizeof(int32_t) * (size_t)nc);
    const size_t b_tiles = round256(sizeof(GrawaTile) * (size_t)bound);
    const size_t b_lt0 = round256(sizeof(int32_t) * ((size_t)L + 1));
    const size_t b_part = round256(sizeof(double) * (size_t)K * (size_t)bound);
    const size_t b_S = round256(sizeof(double) * (size_t)K * (size_t)L);
    const size_t b_A = round256(sizeof(float) * (size_t)K * (size_t)L);
    const size_t b_bm = round256(sizeof(float) * (size_t)K);
    if (b_cells + b_tiles + b_lt0 + b_part + b_S + 2 * b_A + b_bm > GRAWA_STATIC_SCRATCH_BYTES)
        return GRAWA_ERR_UNSUPPORTED; // the problem needs more scratch than the fixed array holds

    int dev = -1;
    void *base = nullptr;
    if (scratch_of_current_device(&dev, &base) != hipSuccess) return GRAWA_ERR_HIP;

    grawa_plan p;
    std::memset(&p, 0, sizeof(p));
    p.K = K;
    p.L = L;
    p.P = P;
    p.tile_elems = T;
    p.n_tiles = bound;
    p.n_cells = nc;
    p.device = dev;
    char *w = static_cast<char *>(base);
    p.d_off = const_cast<int64_t *>(layer_offsets_dev); // read only
    p.d_cell_layer = reinterpret_cast<int32_t *>(w); w += b_cells;
    p.d_tiles = reinterpret_cast<GrawaTile *>(w); w += b_tiles;
    p.d_layer_tile0 = reinterpret_cast<int32_t *>(w); w += b_lt0;
    p.d_partials = reinterpret_cast<double *>(w); w += b_part;
    p.d_S = reinterpret_cast<double *>(w); w += b_S;
    p.d_A = reinterpret_cast<float *>(w); w += b_A;
    p.d_beta_layer = reinterpret_cast<float *>(w); w += b_A;
    p.d_beta_model = reinterpret_cast<float *>(w);

    // Nothing in the scratch has to start at zero: the maps, every partial (K x bound) and the
    // K x L tables are written in full before they are read.
    hipStream_t s = static_cast<hipStream_t>(stream);
    k_static_layer_tiles<<<dim3(1), dim3(GRAWA_SCAN_BLOCK), 0, s>>>(layer_offsets_dev, L, P, T, bound,
                                                                  p.d_layer_tile0);
    if (hipGetLastError() != hipSuccess) return GRAWA_ERR_HIP;
    const int64_t n_map = bound > nc ? bound : nc;
    k_static_maps<<<dim3((unsigned)((n_map + GRAWA_BLOCK - 1) / GRAWA_BLOCK)), dim3(GRAWA_BLOCK), 0, s>>>(
        layer_offsets_dev, L, P, T, bound, p.d_layer_tile0, p.d_tiles, nc, p.d_cell_layer);
    if (hipGetLastError() != hipSuccess) return GRAWA_ERR_HIP;
    if (grawa_launch_sumsq(&p, g, ldg, dt, s, nullptr, nullptr) != hipSuccess) return GRAWA_ERR_HIP;
    if (grawa_launch_finalize_layers(&p, nullptr, weights_out, s, 0, 0.0) != hipSuccess) return GRAWA_ERR_HIP;
    if (grawa_launch_center_pull(&p, x, ldx, p.d_beta_layer, 1, lambda, nullptr, 0, GRAWA_F32, 0.f, 0, center_out,
                                 0.f, 0, s, nullptr, nullptr) != hipSuccess)
        return GRAWA_ERR_HIP;
    return GRAWA_OK;
}
