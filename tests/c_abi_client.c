/*
 * A plain C99 caller of the library (no Python, no torch): builds a small seeded problem, runs
 *   grawa_local_sgd -> grawa_lgrawa_update -> grawa_mgrawa_update_sgd
 * through the C ABI of include/grawa.h and prints the weights and the updated parameters, which a
 * test compares with the CPU reference on the same inputs; then runs grawa_lgrawa_update and
 * grawa_lgrawa_update_static (no plan, no allocation, layer offsets in device memory) on fresh copies
 * of the inputs and reports whether the two agree bit for bit, and what grawa_plan_nonfinite reads
 * (nothing non-finite was seen).  Inputs come from a 32-bit linear
 * congruential generator (x_{n+1} = 1664525 x_n + 1013904223) that the test restates.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "grawa.h"

#define K 3
#define L 4
static const int64_t SIZES[L] = {5, 300, 1, 1000};

static uint32_t state = 12345u;
static float draw(void)
{
    state = 1664525u * state + 1013904223u;
    return (float)((state >> 8) & 0xFFFFu) / 65536.0f - 0.5f; /* multiples of 2^-16 in [-0.5, 0.5) */
}

#define HIP_OK(call)                                                            \
    do {                                                                        \
        hipError_t e_ = (call);                                                 \
        if (e_ != hipSuccess) {                                                 \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));   \
            return 2;                                                           \
        }                                                                       \
    } while (0)
#define GRAWA_OK_OR_DIE(call)                                                            \
    do {                                                                                 \
        grawa_status_t s_ = (call);                                                      \
        if (s_ != GRAWA_OK) {                                                            \
            fprintf(stderr, "%s failed: %s\n", #call, grawa_status_string(s_));          \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

int main(void)
{
    int64_t off[L + 1];
    off[0] = 0;
    for (int l = 0; l < L; ++l) off[l + 1] = off[l] + SIZES[l];
    const int64_t P = off[L], ld = (P + 7) / 8 * 8;
    float *hx = (float *)malloc(sizeof(float) * K * ld), *hg = (float *)malloc(sizeof(float) * K * ld);
    float hb[K * L], hbm[K];
    if (!hx || !hg) return 1;
    for (int k = 0; k < K; ++k)
        for (int64_t i = 0; i < ld; ++i) {
            hx[k * ld + i] = draw();
            hg[k * ld + i] = draw() * (float)(1 << (2 * k)); /* worker k's gradients are 4^k times larger */
        }
    float *hx0 = (float *)malloc(sizeof(float) * K * ld), *hx2 = (float *)malloc(sizeof(float) * K * ld);
    if (!hx0 || !hx2) return 1;
    memcpy(hx0, hx, sizeof(float) * K * ld);
    float *dx, *dg, *db, *dbm, *dc;
    HIP_OK(hipMalloc((void **)&dx, sizeof(float) * K * ld));
    HIP_OK(hipMalloc((void **)&dg, sizeof(float) * K * ld));
    HIP_OK(hipMalloc((void **)&db, sizeof(float) * K * L));
    HIP_OK(hipMalloc((void **)&dbm, sizeof(float) * K));
    HIP_OK(hipMalloc((void **)&dc, sizeof(float) * ld));
    HIP_OK(hipMemcpy(dx, hx, sizeof(float) * K * ld, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dg, hg, sizeof(float) * K * ld, hipMemcpyHostToDevice));

    grawa_plan_t *plan = NULL;
    GRAWA_OK_OR_DIE(grawa_plan_create(&plan, K, P, L, off));
    GRAWA_OK_OR_DIE(grawa_local_sgd(dx, ld, dg, ld, GRAWA_F32, K, P, 0.125f, NULL));
    GRAWA_OK_OR_DIE(grawa_lgrawa_update(plan, dx, ld, dg, ld, GRAWA_F32, 0.25f, dc, db, NULL));
    GRAWA_OK_OR_DIE(grawa_mgrawa_update_sgd(plan, dx, ld, dg, ld, GRAWA_F32, GRAWA_NORM_LAYERSUM, 0.5f, dg, ld,
                                            0.0625f, NULL, dbm, NULL));
    /* an error must come back as a code and leave everything as it is */
    if (grawa_lgrawa_update(plan, dx, ld, dg, ld, GRAWA_F32, 1.5f, NULL, NULL, NULL) != GRAWA_ERR_INVALID_ARG) return 4;
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(hx, dx, sizeof(float) * K * ld, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hb, db, sizeof(float) * K * L, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hbm, dbm, sizeof(float) * K, hipMemcpyDeviceToHost));

    /* plan-based and allocation-free LGRAWA update on the same fresh inputs */
    float *dx2, *dx3, *db2, *db3, hb2[K * L], hb3[K * L];
    int64_t *doff;
    unsigned flags = 99u;
    HIP_OK(hipMalloc((void **)&dx2, sizeof(float) * K * ld));
    HIP_OK(hipMalloc((void **)&dx3, sizeof(float) * K * ld));
    HIP_OK(hipMalloc((void **)&db2, sizeof(float) * K * L));
    HIP_OK(hipMalloc((void **)&db3, sizeof(float) * K * L));
    HIP_OK(hipMalloc((void **)&doff, sizeof(int64_t) * (L + 1)));
    HIP_OK(hipMemcpy(dx2, hx0, sizeof(float) * K * ld, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dx3, hx0, sizeof(float) * K * ld, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(doff, off, sizeof(int64_t) * (L + 1), hipMemcpyHostToDevice));
    GRAWA_OK_OR_DIE(grawa_lgrawa_update(plan, dx2, ld, dg, ld, GRAWA_F32, 0.25f, NULL, db2, NULL));
    GRAWA_OK_OR_DIE(grawa_lgrawa_update_static(K, P, L, doff, dx3, ld, dg, ld, GRAWA_F32, 0.25f, NULL, db3, NULL));
    GRAWA_OK_OR_DIE(grawa_plan_nonfinite(plan, &flags, 1, NULL));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(hx0, dx2, sizeof(float) * K * ld, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hx2, dx3, sizeof(float) * K * ld, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hb2, db2, sizeof(float) * K * L, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hb3, db3, sizeof(float) * K * L, hipMemcpyDeviceToHost));
    const int same = memcmp(hx0, hx2, sizeof(float) * K * ld) == 0 && memcmp(hb2, hb3, sizeof hb2) == 0;
    GRAWA_OK_OR_DIE(grawa_plan_destroy(plan));

    printf("P %lld ld %lld\n", (long long)P, (long long)ld);
    printf("static_equal %d\n", same);
    printf("nonfinite %u\n", flags);
    for (int i = 0; i < K * L; ++i) printf("beta_layer %.9g\n", hb[i]);
    for (int k = 0; k < K; ++k) printf("beta_model %.9g\n", hbm[k]);
    for (int k = 0; k < K; ++k)
        for (int64_t i = 0; i < ld; ++i) printf("x %.9g\n", hx[k * ld + i]);
    HIP_OK(hipFree(dx));
    HIP_OK(hipFree(dg));
    HIP_OK(hipFree(db));
    HIP_OK(hipFree(dbm));
    HIP_OK(hipFree(dc));
    HIP_OK(hipFree(dx2));
    HIP_OK(hipFree(dx3));
    HIP_OK(hipFree(db2));
    HIP_OK(hipFree(db3));
    HIP_OK(hipFree(doff));
    free(hx);
    free(hg);
    free(hx0);
    free(hx2);
    return 0;
}
