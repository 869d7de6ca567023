// Host side of the C ABI declared in include/grawa.h: argument checks, the plan (tile map
// and workspace) and the launch sequence of each entry point.  Nothing here computes any
// part of the update; every step runs in the kernels of grawa_norms.hip, grawa_pull.hip and grawa_local.hip.
#include <cmath>
#include <cstring>
#include <new>

#include "grawa_internal.h"

namespace {

inline size_t round256(size_t n) { return (n + 255) & ~size_t(255); }

grawa_status_t check_params(const grawa_plan *p, const float *x, int64_t ldx)
{
    if (!p) return GRAWA_ERR_INVALID_ARG;
    return grawa_check_params(p->P, x, ldx);
}

inline grawa_status_t check_grads(int64_t P, const void *g, int64_t ldg, grawa_dtype_t dt)
{
    return grawa_check_grads(P, g, ldg, dt);
}
inline grawa_status_t check_lambda(float lambda) { return grawa_check_lambda(lambda); }
inline grawa_status_t check_center(const float *c) { return grawa_check_center(c); }
inline bool aligned16(const void *p) { return grawa_aligned16(p); }

struct DeviceGuard { // the plan's kernels run on the device the plan was made on
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
    }
    ~DeviceGuard()
    {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

// Event bookkeeping for the measurement aid: a profiled call takes one slot of four events and
// notes whether its norm-kernel pair was recorded.
inline bool prof_active(const grawa_plan *p) { return p->profile_on && p->profile_n < GRAWA_PROFILE_SLOTS; }
inline void prof_commit(grawa_plan *p, bool with_norm)
{
    p->ev_norm[p->profile_n] = with_norm ? 1 : 0;
    p->profile_n += 1;
}

#define GRAWA_TRY_HIP(expr)                       \
    do {                                          \
        if ((expr) != hipSuccess) return GRAWA_ERR_HIP; \
    } while (0)

// norms -> weights -> (sgd) center pull; shared by the four update entry points.
grawa_status_t run_update(grawa_plan *p, float *x, int64_t ldx, const void *g, int64_t ldg,
                          grawa_dtype_t dt, int per_layer, grawa_norm_mode_t mode, float lambda,
                          const void *g_sgd, int64_t ldg_sgd, float lr, int fuse_sgd, float *center_out,
                          float *weights_out, hipStream_t s)
{
    grawa_status_t st;
    if ((st = check_params(p, x, ldx)) != GRAWA_OK) return st;
    if ((st = check_grads(p->P, g, ldg, dt)) != GRAWA_OK) return st;
    if ((st = check_lambda(lambda)) != GRAWA_OK) return st;
    if ((st = check_center(center_out)) != GRAWA_OK) return st;
    if (mode != GRAWA_NORM_LAYERSUM && mode != GRAWA_NORM_FLAT) return GRAWA_ERR_INVALID_ARG;
    if (fuse_sgd) {
        if ((st = check_grads(p->P, g_sgd, ldg_sgd, dt)) != GRAWA_OK) return st;
        if (!std::isfinite(lr)) return GRAWA_ERR_INVALID_ARG;
    }
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;

    const bool prof = prof_active(p);
    hipEvent_t *ev = prof ? p->ev + 4 * (size_t)p->profile_n : nullptr;

    GRAWA_TRY_HIP(grawa_launch_sumsq(p, g, ldg, dt, s, prof ? ev[0] : nullptr, prof ? ev[1] : nullptr));

    GRAWA_TRY_HIP(grawa_launch_finalize_layers(p, nullptr, per_layer ? weights_out : nullptr, s, 0, 0.0));
    if (!per_layer) GRAWA_TRY_HIP(grawa_launch_finalize_model(p, mode, weights_out, s));

    GRAWA_TRY_HIP(grawa_launch_center_pull(p, x, ldx, per_layer ? p->d_beta_layer : p->d_beta_model,
                                           per_layer, lambda, g_sgd, ldg_sgd, dt, lr, fuse_sgd,
                                           center_out, 0.f, 0, s, prof ? ev[2] : nullptr, prof ? ev[3] : nullptr));
    if (prof) prof_commit(p, true);
    return GRAWA_OK;
}

} // namespace

extern "C" {

const char *grawa_status_string(grawa_status_t s)
{
    switch (s) {
    case GRAWA_OK: return "ok";
    case GRAWA_ERR_INVALID_ARG: return "invalid argument";
    case GRAWA_ERR_ALIGNMENT: return "pointer or leading dimension not 16-byte aligned";
    case GRAWA_ERR_WORKSPACE: return "workspace allocation failed";
    case GRAWA_ERR_UNSUPPORTED: return "unsupported size or dtype";
    case GRAWA_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

static grawa_status_t plan_create_impl(grawa_plan_t **out, int K, int64_t P, int L,
                                       const int64_t *layer_offsets_host);

grawa_status_t grawa_plan_create(grawa_plan_t **out, int K, int64_t P, int L,
                                 const int64_t *layer_offsets_host)
{
    try { // the host-side maps live in std::vector; no exception may cross the C boundary
        return plan_create_impl(out, K, P, L, layer_offsets_host);
    } catch (...) {
        if (out) *out = nullptr;
        return GRAWA_ERR_WORKSPACE;
    }
}

static grawa_status_t plan_create_impl(grawa_plan_t **out, int K, int64_t P, int L,
                                       const int64_t *layer_offsets_host)
{
    if (!out) return GRAWA_ERR_INVALID_ARG;
    *out = nullptr;
    if (K < 1 || P < 1 || L < 1 || (int64_t)L > P) return GRAWA_ERR_INVALID_ARG;
    if (!layer_offsets_host && L != 1) return GRAWA_ERR_INVALID_ARG;
    if (K > GRAWA_MAX_WORKERS) return GRAWA_ERR_UNSUPPORTED;

    int64_t whole[2] = {0, P};
    const int64_t *off = layer_offsets_host ? layer_offsets_host : whole;
    if (grawa_offsets_invalid(P, L, off)) return GRAWA_ERR_INVALID_ARG;

    const int T = grawa_default_tile_elems(K, P);
    GrawaHostMaps m;
    if (grawa_build_maps(P, L, off, T, m)) return GRAWA_ERR_UNSUPPORTED;
    const int64_t nt = (int64_t)m.tiles.size();
    const int64_t nrt = (int64_t)m.rtiles.size();
    const int64_t nrb = (int64_t)m.block_rtile0.size() - 1;
    const int64_t nc = (int64_t)m.cell_layer.size();

    grawa_plan *p = new (std::nothrow) grawa_plan();
    if (!p) return GRAWA_ERR_WORKSPACE;
    std::memset(p, 0, sizeof(*p));
    p->K = K;
    p->L = L;
    p->P = P;
    p->tile_elems = T;
    p->n_tiles = nt;
    p->n_rtiles = nrt;
    p->n_cells = nc;
    if (hipGetDevice(&p->device) != hipSuccess) {
        delete p;
        return GRAWA_ERR_HIP;
    }

    const size_t b_off = round256(sizeof(int64_t) * ((size_t)L + 1));
    const size_t b_cells = round256(sizeof(int32_t) * (size_t)nc);
    const size_t b_tiles = round256(sizeof(GrawaTile) * (size_t)nt);
    const size_t b_rtiles = round256(sizeof(GrawaTile) * (size_t)nrt);
    const size_t b_lt0 = round256(sizeof(int32_t) * ((size_t)L + 1));
    const size_t b_brt0 = round256(sizeof(int32_t) * ((size_t)nrb + 1));
    const size_t b_part = round256(sizeof(double) * (size_t)K * (size_t)(nrt > nt ? nrt : nt));
    const size_t b_S = round256(sizeof(double) * (size_t)K * (size_t)L);
    const size_t b_A = round256(sizeof(float) * (size_t)K * (size_t)L);
    const size_t b_bl = b_A;
    const size_t b_bm = round256(sizeof(float) * (size_t)K);
    const size_t b_mvg = b_S;
    const size_t b_t = 256;
    p->ws_bytes = b_off + b_cells + b_tiles + b_lt0 + b_rtiles + b_lt0 + b_brt0 + b_part + b_S + b_A + b_bl + b_bm + b_mvg + b_t;
    if (hipMalloc(&p->ws, p->ws_bytes) != hipSuccess) {
        (void)hipGetLastError();
        delete p;
        return GRAWA_ERR_WORKSPACE;
    }
    char *w = static_cast<char *>(p->ws);
    p->d_off = reinterpret_cast<int64_t *>(w); w += b_off;
    p->d_cell_layer = reinterpret_cast<int32_t *>(w); w += b_cells;
    p->d_tiles = reinterpret_cast<GrawaTile *>(w); w += b_tiles;
    p->d_layer_tile0 = reinterpret_cast<int32_t *>(w); w += b_lt0;
    p->d_rtiles = reinterpret_cast<GrawaTile *>(w); w += b_rtiles;
    p->d_layer_rtile0 = reinterpret_cast<int32_t *>(w); w += b_lt0;
    p->d_block_rtile0 = reinterpret_cast<int32_t *>(w); w += b_brt0;
    p->d_partials = reinterpret_cast<double *>(w); w += b_part;
    p->d_S = reinterpret_cast<double *>(w); w += b_S;
    p->d_A = reinterpret_cast<float *>(w); w += b_A;
    p->d_beta_layer = reinterpret_cast<float *>(w); w += b_bl;
    p->d_beta_model = reinterpret_cast<float *>(w); w += b_bm;
    p->d_mvg = reinterpret_cast<double *>(w); w += b_mvg;
    p->d_local_t = reinterpret_cast<int64_t *>(w);
    p->d_flags = reinterpret_cast<unsigned *>(w + 64);

    if (hipMemcpy(p->d_off, off, sizeof(int64_t) * ((size_t)L + 1), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_cell_layer, m.cell_layer.data(), sizeof(int32_t) * (size_t)nc, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_tiles, m.tiles.data(), sizeof(GrawaTile) * (size_t)nt, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_layer_tile0, m.layer_tile0.data(), sizeof(int32_t) * ((size_t)L + 1), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_rtiles, m.rtiles.data(), sizeof(GrawaTile) * (size_t)nrt, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_layer_rtile0, m.layer_rtile0.data(), sizeof(int32_t) * ((size_t)L + 1), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_block_rtile0, m.block_rtile0.data(), sizeof(int32_t) * ((size_t)nrb + 1), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemset(p->d_partials, 0, b_part + b_S + b_A + b_bl + b_bm + b_mvg + b_t) != hipSuccess) {
        (void)hipFree(p->ws);
        delete p;
        return GRAWA_ERR_HIP;
    }
    *out = p;
    return GRAWA_OK;
}

grawa_status_t grawa_plan_destroy(grawa_plan_t *p)
{
    if (!p) return GRAWA_OK;
    grawa_status_t st = GRAWA_OK;
    if (p->ev) {
        for (int i = 0; i < 4 * GRAWA_PROFILE_SLOTS; ++i)
            if (p->ev[i]) (void)hipEventDestroy(p->ev[i]);
        delete[] p->ev;
        delete[] p->ev_norm;
    }
    if (p->ws && hipFree(p->ws) != hipSuccess) st = GRAWA_ERR_HIP;
    delete p;
    return st;
}

grawa_status_t grawa_plan_info(const grawa_plan_t *p, int64_t *n_tiles, int *tile_elems)
{
    if (!p) return GRAWA_ERR_INVALID_ARG;
    if (n_tiles) *n_tiles = p->n_tiles;
    if (tile_elems) *tile_elems = p->tile_elems;
    return GRAWA_OK;
}

grawa_status_t grawa_grad_norms(grawa_plan_t *p, const void *g, int64_t ldg, grawa_dtype_t dt,
                                float *norms_out, void *stream)
{
    if (!p || !norms_out) return GRAWA_ERR_INVALID_ARG;
    grawa_status_t st = check_grads(p->P, g, ldg, dt);
    if (st != GRAWA_OK) return st;
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GRAWA_TRY_HIP(grawa_launch_sumsq(p, g, ldg, dt, s, nullptr, nullptr));
    GRAWA_TRY_HIP(grawa_launch_finalize_layers(p, norms_out, nullptr, s, 0, 0.0));
    return GRAWA_OK;
}

grawa_status_t grawa_mgrawa_update(grawa_plan_t *p, float *x, int64_t ldx, const void *g, int64_t ldg,
                                   grawa_dtype_t dt, grawa_norm_mode_t mode, float lambda,
                                   float *center_out, float *weights_out, void *stream)
{
    return run_update(p, x, ldx, g, ldg, dt, 0, mode, lambda, nullptr, 0, 0.f, 0, center_out, weights_out,
                      static_cast<hipStream_t>(stream));
}

grawa_status_t grawa_lgrawa_update(grawa_plan_t *p, float *x, int64_t ldx, const void *g, int64_t ldg,
                                   grawa_dtype_t dt, float lambda, float *center_out, float *weights_out,
                                   void *stream)
{
    return run_update(p, x, ldx, g, ldg, dt, 1, GRAWA_NORM_LAYERSUM, lambda, nullptr, 0, 0.f, 0, center_out,
                      weights_out, static_cast<hipStream_t>(stream));
}

grawa_status_t grawa_mgrawa_update_sgd(grawa_plan_t *p, float *x, int64_t ldx, const void *g, int64_t ldg,
                                       grawa_dtype_t dt, grawa_norm_mode_t mode, float lambda,
                                       const void *g_sgd, int64_t ldg_sgd, float lr, float *center_out,
                                       float *weights_out, void *stream)
{
    return run_update(p, x, ldx, g, ldg, dt, 0, mode, lambda, g_sgd, ldg_sgd, lr, 1, center_out, weights_out,
                      static_cast<hipStream_t>(stream));
}

grawa_status_t grawa_lgrawa_update_sgd(grawa_plan_t *p, float *x, int64_t ldx, const void *g, int64_t ldg,
                                       grawa_dtype_t dt, float lambda, const void *g_sgd, int64_t ldg_sgd,
                                       float lr, float *center_out, float *weights_out, void *stream)
{
    return run_update(p, x, ldx, g, ldg, dt, 1, GRAWA_NORM_LAYERSUM, lambda, g_sgd, ldg_sgd, lr, 1, center_out,
                      weights_out, static_cast<hipStream_t>(stream));
}

grawa_status_t grawa_center_pull(grawa_plan_t *p, float *x, int64_t ldx, const float *weights, int per_layer,
                                 float lambda, float *center_out, void *stream)
{
    grawa_status_t st;
    if ((st = check_params(p, x, ldx)) != GRAWA_OK) return st;
    if (!weights) return GRAWA_ERR_INVALID_ARG;
    if ((st = check_lambda(lambda)) != GRAWA_OK) return st;
    if ((st = check_center(center_out)) != GRAWA_OK) return st;
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool prof = prof_active(p);
    hipEvent_t *ev = prof ? p->ev + 4 * (size_t)p->profile_n : nullptr;
    GRAWA_TRY_HIP(grawa_launch_center_pull(p, x, ldx, weights, per_layer ? 1 : 0, lambda, nullptr, 0, GRAWA_F32,
                                           0.f, 0, center_out, 0.f, 0, s, prof ? ev[2] : nullptr,
                                           prof ? ev[3] : nullptr));
    if (prof) prof_commit(p, false);
    return GRAWA_OK;
}

grawa_status_t grawa_local_sgd(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt, int K,
                               int64_t P, float lr, void *stream)
{
    if (!x || K < 1 || P < 1 || ldx < P) return GRAWA_ERR_INVALID_ARG;
    if (K > 65535 || P >= ((int64_t)1 << 32)) return GRAWA_ERR_UNSUPPORTED; /* grid.y; 2^22 column blocks */
    if (!aligned16(x) || (ldx % 4) != 0) return GRAWA_ERR_ALIGNMENT;
    grawa_status_t st = check_grads(P, g, ldg, dt);
    if (st != GRAWA_OK) return st;
    if (!std::isfinite(lr)) return GRAWA_ERR_INVALID_ARG;
    GRAWA_TRY_HIP(grawa_launch_row_step(x, ldx, g, ldg, dt, lr, nullptr, 0.f, K, P, nullptr, nullptr, 0, nullptr,
                                        static_cast<hipStream_t>(stream)));
    return GRAWA_OK;
}

grawa_status_t grawa_local_nesterov(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt, float *buf,
                                    int64_t ldb, int K, int64_t P, float lr, float momentum, float weight_decay,
                                    void *stream)
{
    if (!x || !buf || K < 1 || P < 1 || ldx < P || ldb < P) return GRAWA_ERR_INVALID_ARG;
    if (K > 65535 || P >= ((int64_t)1 << 32)) return GRAWA_ERR_UNSUPPORTED;
    if (!aligned16(x) || (ldx % 4) != 0 || !aligned16(buf) || (ldb % 4) != 0) return GRAWA_ERR_ALIGNMENT;
    grawa_status_t st = check_grads(P, g, ldg, dt);
    if (st != GRAWA_OK) return st;
    if (!std::isfinite(lr) || !std::isfinite(momentum) || !std::isfinite(weight_decay) || momentum < 0.f ||
        weight_decay < 0.f)
        return GRAWA_ERR_INVALID_ARG;
    GRAWA_TRY_HIP(grawa_launch_nesterov(x, ldx, g, ldg, dt, buf, ldb, K, P, lr, momentum, weight_decay,
                                        static_cast<hipStream_t>(stream)));
    return GRAWA_OK;
}

/* EASGD and LSGD share the pull kernel: only the weights (and the moving center) differ. */
static grawa_status_t run_fixed_center(grawa_plan_t *p, float *x, int64_t ldx, const float *loss, float lambda,
                                       float rho, int moving, float *center, float *weights_out, int *leader_out,
                                       void *stream)
{
    grawa_status_t st;
    if ((st = check_params(p, x, ldx)) != GRAWA_OK) return st;
    if ((st = check_lambda(lambda)) != GRAWA_OK) return st;
    if ((st = check_center(center)) != GRAWA_OK) return st;
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GRAWA_TRY_HIP(grawa_launch_center_weights(p, loss, weights_out, leader_out, s));
    GRAWA_TRY_HIP(grawa_launch_center_pull(p, x, ldx, p->d_beta_model, 0, lambda, nullptr, 0, GRAWA_F32, 0.f, 0,
                                           center, rho, moving, s, nullptr, nullptr));
    return GRAWA_OK;
}

grawa_status_t grawa_easgd_update(grawa_plan_t *p, float *x, int64_t ldx, float lambda, float rho, float *center,
                                  void *stream)
{
    if (!center || !(rho >= 0.f && rho <= 1.f)) return GRAWA_ERR_INVALID_ARG;
    return run_fixed_center(p, x, ldx, nullptr, lambda, rho, 1, center, nullptr, nullptr, stream);
}

grawa_status_t grawa_lsgd_update(grawa_plan_t *p, float *x, int64_t ldx, const float *losses, float lambda,
                                 float *center_out, int *leader_out, void *stream)
{
    if (!losses) return GRAWA_ERR_INVALID_ARG;
    return run_fixed_center(p, x, ldx, losses, lambda, 0.f, 0, center_out, nullptr, leader_out, stream);
}

grawa_status_t grawa_local_sgd_prox(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt, int K,
                                    int64_t P, float lr, const float *center, float mu, float tau, void *stream)
{
    if (!x || !center || K < 1 || P < 1 || ldx < P) return GRAWA_ERR_INVALID_ARG;
    if (K > 65535 || P >= ((int64_t)1 << 32)) return GRAWA_ERR_UNSUPPORTED; /* grid.y; 2^22 column blocks */
    if (!aligned16(x) || (ldx % 4) != 0 || !aligned16(center)) return GRAWA_ERR_ALIGNMENT;
    grawa_status_t st = check_grads(P, g, ldg, dt);
    if (st != GRAWA_OK) return st;
    if (!std::isfinite(lr) || !std::isfinite(mu) || !std::isfinite(tau) || !(tau > 0.f) || mu < 0.f || mu > tau)
        return GRAWA_ERR_INVALID_ARG;
    GRAWA_TRY_HIP(grawa_launch_row_step(x, ldx, g, ldg, dt, lr, center, mu / tau, K, P, nullptr, nullptr, 0, nullptr,
                                        static_cast<hipStream_t>(stream)));
    return GRAWA_OK;
}

grawa_status_t grawa_local_step_scored(grawa_plan_t *p, float *x, int64_t ldx, const void *g, int64_t ldg,
                                       grawa_dtype_t dt, float lr, const float *center, float mu, float tau,
                                       float gamma, void *stream)
{
    grawa_status_t st;
    if ((st = check_params(p, x, ldx)) != GRAWA_OK) return st;
    if ((st = check_grads(p->P, g, ldg, dt)) != GRAWA_OK) return st;
    if (!std::isfinite(lr) || !(gamma > 0.f) || !(gamma < 1.f)) return GRAWA_ERR_INVALID_ARG;
    if (p->local_t > 0 && (double)gamma != p->local_gamma) return GRAWA_ERR_INVALID_ARG; /* one gamma per round */
    float w = 0.f;
    if (center) {
        if (!aligned16(center)) return GRAWA_ERR_ALIGNMENT;
        if (!std::isfinite(mu) || !std::isfinite(tau) || !(tau > 0.f) || mu < 0.f || mu > tau)
            return GRAWA_ERR_INVALID_ARG;
        w = mu / tau;
    }
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GRAWA_TRY_HIP(grawa_launch_row_step(x, ldx, g, ldg, dt, lr, center, w, p->K, p->P, p->d_rtiles,
                                        p->d_block_rtile0, p->n_rtiles, p->d_partials, s));
    GRAWA_TRY_HIP(grawa_launch_finalize_layers(p, nullptr, nullptr, s, 1, (double)gamma));
    p->local_t += 1;
    p->local_gamma = (double)gamma;
    return GRAWA_OK;
}

namespace {
grawa_status_t local_update(grawa_plan_t *p, float *x, int64_t ldx, int per_layer, float lambda, float *center_out,
                            float *weights_out, float *est_out, hipStream_t s)
{
    grawa_status_t st;
    if ((st = check_params(p, x, ldx)) != GRAWA_OK) return st;
    if ((st = check_lambda(lambda)) != GRAWA_OK) return st;
    if ((st = check_center(center_out)) != GRAWA_OK) return st;
    if (p->local_t < 1) return GRAWA_ERR_INVALID_ARG; /* no local step since the last communication */
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    GRAWA_TRY_HIP(grawa_launch_local_weights(p, p->local_gamma, per_layer, weights_out, est_out, s));
    const bool prof = prof_active(p);
    hipEvent_t *ev = prof ? p->ev + 4 * (size_t)p->profile_n : nullptr;
    GRAWA_TRY_HIP(grawa_launch_center_pull(p, x, ldx, per_layer ? p->d_beta_layer : p->d_beta_model, per_layer,
                                           lambda, nullptr, 0, GRAWA_F32, 0.f, 0, center_out, 0.f, 0, s,
                                           prof ? ev[2] : nullptr, prof ? ev[3] : nullptr));
    if (prof) prof_commit(p, false);
    GRAWA_TRY_HIP(grawa_launch_zero_estimate(p, s));
    p->local_t = 0;
    return GRAWA_OK;
}
} // namespace

grawa_status_t grawa_local_lgrawa_update(grawa_plan_t *p, float *x, int64_t ldx, float lambda, float *center_out,
                                         float *weights_out, float *est_out, void *stream)
{
    return local_update(p, x, ldx, 1, lambda, center_out, weights_out, est_out, static_cast<hipStream_t>(stream));
}

grawa_status_t grawa_local_mgrawa_update(grawa_plan_t *p, float *x, int64_t ldx, float lambda, float *center_out,
                                         float *weights_out, float *est_out, void *stream)
{
    return local_update(p, x, ldx, 0, lambda, center_out, weights_out, est_out, static_cast<hipStream_t>(stream));
}

grawa_status_t grawa_local_scores_reset(grawa_plan_t *p, void *stream)
{
    if (!p) return GRAWA_ERR_INVALID_ARG;
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    GRAWA_TRY_HIP(grawa_launch_zero_estimate(p, static_cast<hipStream_t>(stream)));
    p->local_t = 0;
    p->local_gamma = 0.0;
    return GRAWA_OK;
}

grawa_status_t grawa_plan_nonfinite(grawa_plan_t *p, unsigned *flags_host, int clear, void *stream)
{
    if (!p || !flags_host) return GRAWA_ERR_INVALID_ARG;
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GRAWA_TRY_HIP(hipStreamSynchronize(s));
    GRAWA_TRY_HIP(hipMemcpy(flags_host, p->d_flags, sizeof(unsigned), hipMemcpyDeviceToHost));
    if (clear) GRAWA_TRY_HIP(grawa_launch_clear_flags(p, s));
    return GRAWA_OK;
}

grawa_status_t grawa_plan_profile(grawa_plan_t *p, int enable)
{
    if (!p) return GRAWA_ERR_INVALID_ARG;
    DeviceGuard guard(p->device);
    if (!guard.ok) return GRAWA_ERR_HIP;
    if (enable && !p->ev) {
        const int n = 4 * GRAWA_PROFILE_SLOTS;
        hipEvent_t *ev = new (std::nothrow) hipEvent_t[n]();
        unsigned char *flags = new (std::nothrow) unsigned char[GRAWA_PROFILE_SLOTS]();
        bool ok = ev && flags;
        for (int i = 0; ok && i < n; ++i) ok = hipEventCreate(&ev[i]) == hipSuccess;
        if (!ok) { // give back whatever was created
            const bool no_mem = !ev || !flags;
            if (ev)
                for (int i = 0; i < n; ++i)
                    if (ev[i]) (void)hipEventDestroy(ev[i]);
            delete[] ev;
            delete[] flags;
            return no_mem ? GRAWA_ERR_WORKSPACE : GRAWA_ERR_HIP;
        }
        p->ev = ev;
        p->ev_norm = flags;
    }
    p->profile_on = enable ? 1 : 0;
    p->profile_n = 0;
    return GRAWA_OK;
}

grawa_status_t grawa_plan_profile_read(grawa_plan_t *p, int *n_calls, double *norm_ms, double *pull_ms)
{
    if (!p) return GRAWA_ERR_INVALID_ARG;
    double a = 0.0, b = 0.0;
    for (int i = 0; i < p->profile_n; ++i) {
        float ms = 0.f;
        if (p->ev_norm[i]) {
            GRAWA_TRY_HIP(hipEventElapsedTime(&ms, p->ev[4 * i + 0], p->ev[4 * i + 1]));
            a += ms;
        }
        GRAWA_TRY_HIP(hipEventElapsedTime(&ms, p->ev[4 * i + 2], p->ev[4 * i + 3]));
        b += ms;
    }
    if (n_calls) *n_calls = p->profile_n;
    if (norm_ms) *norm_ms = a;
    if (pull_ms) *pull_ms = b;
    return GRAWA_OK;
}

grawa_status_t grawa_plan_profile_read_call(grawa_plan_t *p, int i, double *norm_ms, double *pull_ms, double *span_ms)
{
    if (!p || i < 0 || i >= p->profile_n) return GRAWA_ERR_INVALID_ARG;
    float a = 0.f, b = 0.f, c = 0.f;
    GRAWA_TRY_HIP(hipEventElapsedTime(&b, p->ev[4 * i + 2], p->ev[4 * i + 3]));
    c = b;
    if (p->ev_norm[i]) {
        GRAWA_TRY_HIP(hipEventElapsedTime(&a, p->ev[4 * i + 0], p->ev[4 * i + 1]));
        GRAWA_TRY_HIP(hipEventElapsedTime(&c, p->ev[4 * i + 0], p->ev[4 * i + 3]));
    }
    if (norm_ms) *norm_ms = a;
    if (pull_ms) *pull_ms = b;
    if (span_ms) *span_ms = c;
    return GRAWA_OK;
}

grawa_status_t grawa_stream_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (!dst || !src || nbytes < 0) return GRAWA_ERR_INVALID_ARG;
    if (!aligned16(dst) || !aligned16(src) || (nbytes % 16) != 0) return GRAWA_ERR_ALIGNMENT;
    if (nbytes / 16 >= ((int64_t)1 << 32)) return GRAWA_ERR_UNSUPPORTED; /* grid.x * 64 < 2^32 */
    GRAWA_TRY_HIP(grawa_launch_stream_copy(dst, src, nbytes, static_cast<hipStream_t>(stream)));
    return GRAWA_OK;
}

} // extern "C"
