// Internal declarations shared by the host API (grawa_api.cpp) and the kernel files
// (grawa_norms.hip, grawa_pull.hip, grawa_local.hip).  Not installed; the public ABI is include/grawa.h.
#ifndef GRAWA_INTERNAL_H
#define GRAWA_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>

#include "grawa.h"
#include "grawa_maps.h"

#define GRAWA_PROFILE_SLOTS 4096

struct grawa_plan {
    int K;
    int L;
    int64_t P;
    int tile_elems;
    int64_t n_tiles;
    int64_t n_cells; // ceil(P / 256): blocks of the center+pull pass
    int device;
    // one device allocation, carved up:
    void *ws;
    size_t ws_bytes;
    int64_t *d_off;         // [L+1] layer offsets
    GrawaTile *d_tiles;     // [n_tiles]
    int32_t *d_layer_tile0; // [L+1] first tile of every layer
    GrawaTile *d_rtiles;    // [n_rtiles] short tiles (1024 columns) of the scored local step
    int32_t *d_layer_rtile0; // [L+1]
    int32_t *d_block_rtile0; // [ceil(P/1024)+1] first short tile of every aligned block of 1024 columns
    int64_t n_rtiles;
    int32_t *d_cell_layer;  // [n_cells] layer of a 256-column cell, or ~(first layer) if it holds a boundary
    double *d_partials;     // [K][n_tiles] per-tile sums of squares
    double *d_S;            // [K][L] squared Frobenius norms
    float *d_A;             // [K][L] layer norms
    float *d_beta_layer;    // [K][L] per-layer weights
    float *d_beta_model;    // [K] model-level weights
    double *d_mvg;          // [K][L] moving average of the layer norms (running estimate, Appendix G)
    int64_t *d_local_t;     // device: local steps since the last communication (what the kernels use)
    unsigned *d_flags;      // device: GRAWA_NONFINITE_* bits, sticky until read-and-cleared (may be null)
    int64_t local_t;        // host mirror of the counter as of the last enqueued call (argument checks only)
    double local_gamma;     // momentum of the running estimate used so far (0 = none yet)
    // measurement aid
    int profile_on;
    int profile_n;
    hipEvent_t *ev;          // 4 per slot: norm begin/end, pull begin/end
    unsigned char *ev_norm;  // per slot: 1 if the call recorded norm-kernel events
};

// Argument checks shared by the entry points (host only; nothing is launched on failure).
static inline bool grawa_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline grawa_status_t grawa_check_params(int64_t P, const float *x, int64_t ldx)
{
    if (!x || ldx < P) return GRAWA_ERR_INVALID_ARG;
    if (!grawa_aligned16(x) || (ldx % 4) != 0) return GRAWA_ERR_ALIGNMENT;
    return GRAWA_OK;
}

static inline grawa_status_t grawa_check_grads(int64_t P, const void *g, int64_t ldg, grawa_dtype_t dt)
{
    if (!g) return GRAWA_ERR_INVALID_ARG;
    if (dt != GRAWA_F32 && dt != GRAWA_BF16) return GRAWA_ERR_UNSUPPORTED;
    if (ldg < P) return GRAWA_ERR_INVALID_ARG;
    const int64_t per16 = (dt == GRAWA_BF16) ? 8 : 4;
    if (!grawa_aligned16(g) || (ldg % per16) != 0) return GRAWA_ERR_ALIGNMENT;
    return GRAWA_OK;
}

static inline grawa_status_t grawa_check_lambda(float lambda)
{
    if (!std::isfinite(lambda) || lambda < 0.f || lambda > 1.f) return GRAWA_ERR_INVALID_ARG;
    return GRAWA_OK;
}

static inline grawa_status_t grawa_check_center(const float *c)
{
    if (c && !grawa_aligned16(c)) return GRAWA_ERR_ALIGNMENT;
    return GRAWA_OK;
}

// Launchers (defined next to their kernels).  All return the hipError_t of the launch.
// e0/e1: optional start/stop events of the launch itself (null when not profiling).
hipError_t grawa_launch_sumsq(const grawa_plan *p, const void *g, int64_t ldg, grawa_dtype_t dt,
                              hipStream_t s, hipEvent_t e0, hipEvent_t e1);
hipError_t grawa_launch_finalize_layers(const grawa_plan *p, float *norms_user, float *beta_user,
                                        hipStream_t s, int update_estimate, double gamma);
hipError_t grawa_launch_local_weights(const grawa_plan *p, double gamma, int per_layer, float *beta_user,
                                      float *est_user, hipStream_t s);
hipError_t grawa_launch_zero_estimate(const grawa_plan *p, hipStream_t s);
hipError_t grawa_launch_clear_flags(const grawa_plan *p, hipStream_t s);
hipError_t grawa_launch_row_step(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt, float lr,
                                 const float *center, float w, int K, int64_t P, const GrawaTile *tiles,
                                 const int32_t *block_tile0, int64_t n_tiles, double *partials, hipStream_t s);
hipError_t grawa_launch_finalize_model(const grawa_plan *p, grawa_norm_mode_t mode, float *beta_user,
                                       hipStream_t s);
hipError_t grawa_launch_center_pull(const grawa_plan *p, float *x, int64_t ldx, const float *beta,
                                    int per_layer, float lambda, const void *g_sgd,
                                    int64_t ldg_sgd, grawa_dtype_t dt, float lr, int fuse_sgd,
                                    float *center_out, float rho, int moving, hipStream_t s, hipEvent_t e0,
                                    hipEvent_t e1);
hipError_t grawa_launch_nesterov(float *x, int64_t ldx, const void *g, int64_t ldg, grawa_dtype_t dt,
                                 float *buf, int64_t ldb, int K, int64_t P, float lr, float momentum,
                                 float wd, hipStream_t s);
hipError_t grawa_launch_center_weights(const grawa_plan *p, const float *loss, float *beta_user,
                                       int *leader_out, hipStream_t s);
hipError_t grawa_launch_stream_copy(void *dst, const void *src, int64_t nbytes, hipStream_t s);

#endif
