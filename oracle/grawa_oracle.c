/*
 * grawa_oracle.c -- plain float64 CPU statement of the GRAWA distributed update.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is compared
 * against; it is never part of the product path.  It shares no code, header,
 * table or helper with the HIP library and includes nothing from it.
 *
 * Everything is written as the definition reads: one sequential loop per sum,
 * float64 throughout, inputs (fp32 or bf16 bit patterns) widened exactly per
 * element.  No blocking, no threads, no reordering.
 *
 * Notation (paper -> here): M workers -> K rows; K layers -> L segments given by
 * off[0..L] (off[0]=0, off[L]=P); x_m -> row m of x; G_k of worker m -> the slice
 * off[k]..off[k+1] of row m of g.
 *
 * Sources: vanilla GRAWA weights, Sec. 4.3.1 eq. (2); center and pull, the
 * unnumbered display after eq. (2); MGRAWA, Sec. 5.1 eqs. (3)-(4); LGRAWA,
 * Sec. 5.2 eqs. (5)-(7); local SGD step and its place before the distributed
 * phase, Algorithms 1 and 2; proximity step, same algorithms; running estimate of the
 * norm scores, Appendix G (Local MGRAWA/LGRAWA algorithm); Nesterov-momentum local optimizer,
 * Appendix B.2.2; EASGD and LSGD centers, Appendix F.
 *
 * Every function returns 0 on success, nonzero on a bad argument.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORACLE_F32 0
#define ORACLE_BF16 1

#define ORACLE_NORM_LAYERSUM 0 /* eq. (3): A_m = sum_k ||G_k||_F            */
#define ORACLE_NORM_FLAT 1     /* eq. (2): A_m = || flattened gradient ||_2 */

/* Exact widening of element i of a gradient array to float64.  bfloat16 is the
 * upper 16 bits of an IEEE binary32, so shifting the bits up gives the value. */
static double widen_at(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float *)base)[i];
}

/* Squared Frobenius norm of every (worker, layer) gradient block:
 * S[m*L + k] = sum_{i in layer k} g[m][i]^2   (inner part of eqs. (3) and (5)). */
int oracle_sumsq(const void *g, int dtype, int64_t K, int64_t ldg, int64_t L,
                 const int64_t *off, double *S)
{
    if (!g || !off || !S || K < 1 || L < 1 || ldg < off[L]) return 1;
    for (int64_t m = 0; m < K; ++m) {
        for (int64_t k = 0; k < L; ++k) {
            double s = 0.0;
            for (int64_t i = off[k]; i < off[k + 1]; ++i) {
                double v = widen_at(g, dtype, m * ldg + i);
                s += v * v;
            }
            S[m * L + k] = s;
        }
    }
    return 0;
}

/* LGRAWA scores, eq. (5)-(6): A[m][k] = ||G_k of worker m||_F. */
int oracle_layer_norms(const double *S, int64_t K, int64_t L, double *A)
{
    if (!S || !A || K < 1 || L < 1) return 1;
    for (int64_t m = 0; m < K; ++m)
        for (int64_t k = 0; k < L; ++k)
            A[m * L + k] = sqrt(S[m * L + k]);
    return 0;
}

/* Model-level score per worker.
 * LAYERSUM, eq. (3): A[m] = sum_k ||G_k||_F  (the sum of the layer norms).
 * FLAT, eq. (2):     A[m] = || all of worker m's gradient as one vector ||_2. */
int oracle_model_norms(const double *S, int64_t K, int64_t L, int mode, double *A)
{
    if (!S || !A || K < 1 || L < 1) return 1;
    for (int64_t m = 0; m < K; ++m) {
        double a = 0.0;
        if (mode == ORACLE_NORM_LAYERSUM) {
            for (int64_t k = 0; k < L; ++k) a += sqrt(S[m * L + k]);
        } else if (mode == ORACLE_NORM_FLAT) {
            for (int64_t k = 0; k < L; ++k) a += S[m * L + k];
            a = sqrt(a);
        } else {
            return 2;
        }
        A[m] = a;
    }
    return 0;
}

/* Weights inversely proportional to the scores and summing to one over the
 * workers, eq. (2)/(4)/(7).  A and beta are [K][G]; each of the G columns
 * (G = 1 for the model-level variants, G = L for LGRAWA) is normalised on its
 * own over the worker index.
 *
 * The paper does not say what 1/0 means.  The reading taken is the limit
 * A -> 0+: if n0 >= 1 workers of a column have a score of exactly zero they
 * share the weight equally (1/n0 each) and the others get 0.  A score of +inf
 * gives weight 0 by the same formula; NaN propagates. */
int oracle_weights(const double *A, int64_t K, int64_t G, double *beta)
{
    if (!A || !beta || K < 1 || G < 1) return 1;
    for (int64_t j = 0; j < G; ++j) {
        int64_t n0 = 0;
        for (int64_t m = 0; m < K; ++m)
            if (A[m * G + j] == 0.0) ++n0;
        if (n0 > 0) {
            for (int64_t m = 0; m < K; ++m)
                beta[m * G + j] = (A[m * G + j] == 0.0) ? 1.0 / (double)n0 : 0.0;
            continue;
        }
        double z = 0.0;
        for (int64_t m = 0; m < K; ++m) z += 1.0 / A[m * G + j];
        for (int64_t m = 0; m < K; ++m) beta[m * G + j] = (1.0 / A[m * G + j]) / z;
    }
    return 0;
}

/* Exact widening of the columns [i0, i1) of the fp32 parameter array x[K][ldx]
 * into a dense float64 chunk xd[K][n], n = i1 - i0. */
int oracle_load_params(const float *x, int64_t K, int64_t ldx, int64_t i0, int64_t i1,
                       double *xd)
{
    if (!x || !xd || K < 1 || i0 < 0 || i1 < i0 || ldx < i1) return 1;
    int64_t n = i1 - i0;
    for (int64_t m = 0; m < K; ++m)
        for (int64_t i = 0; i < n; ++i)
            xd[m * n + i] = (double)x[m * ldx + i0 + i];
    return 0;
}

/* Local SGD step of Algorithms 1 and 2 on a chunk: x_m <- x_m - eta * grad_m.
 * xd is the chunk [K][n] holding columns i0.. of the parameters; g is the whole
 * gradient array [K][ldg]. */
int oracle_local_sgd(double *xd, int64_t K, int64_t n, int64_t i0, const void *g,
                     int dtype, int64_t ldg, double eta)
{
    if (!xd || !g || K < 1 || n < 0 || i0 < 0 || ldg < i0 + n) return 1;
    for (int64_t m = 0; m < K; ++m)
        for (int64_t i = 0; i < n; ++i)
            xd[m * n + i] = xd[m * n + i] - eta * widen_at(g, dtype, m * ldg + i0 + i);
    return 0;
}

/* Center variable on a chunk: c[i] = sum_m beta[m][layer(i0+i)] * x_m[i0+i],
 * workers added in index order.  beta is [K][G]; G == 1 means one weight per
 * worker (off may be NULL), otherwise G == L and off[0..L] gives the layers
 * (eq. (7) and the "construct" step that concatenates the layer centers). */
int oracle_center(const double *xd, int64_t K, int64_t n, int64_t i0, const double *beta,
                  int64_t G, const int64_t *off, double *c)
{
    if (!xd || !beta || !c || K < 1 || n < 0 || G < 1 || (G > 1 && !off)) return 1;
    int64_t layer = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (G > 1) {
            while (layer + 1 < G && off[layer + 1] <= i0 + i) ++layer;
        }
        double s = 0.0;
        for (int64_t m = 0; m < K; ++m) s += beta[m * G + layer] * xd[m * n + i];
        c[i] = s;
    }
    return 0;
}

/* Pull of every worker toward the center, written as printed:
 * x_m <- (1 - lambda) x_m + lambda x_C, every worker from its pre-pull value. */
int oracle_pull(double *xd, int64_t K, int64_t n, const double *c, double lambda)
{
    if (!xd || !c || K < 1 || n < 0) return 1;
    for (int64_t m = 0; m < K; ++m)
        for (int64_t i = 0; i < n; ++i)
            xd[m * n + i] = (1.0 - lambda) * xd[m * n + i] + lambda * c[i];
    return 0;
}

/* Proximity step of Algorithms 1 and 2 toward a previously computed center:
 * x_m <- (1 - mu/tau) x_m + (mu/tau) x_C.  c holds the stored center for the
 * same columns as the chunk. */
int oracle_prox(double *xd, int64_t K, int64_t n, const double *c, double mu, double tau)
{
    if (!xd || !c || K < 1 || n < 0 || !(tau > 0.0)) return 1;
    double w = mu / tau;
    for (int64_t m = 0; m < K; ++m)
        for (int64_t i = 0; i < n; ++i)
            xd[m * n + i] = (1.0 - w) * xd[m * n + i] + w * c[i];
    return 0;
}

/* Running estimate of the gradient-norm scores, Appendix G (Local MGRAWA/LGRAWA), one local
 * step for n scores (all workers and layers):
 *     g_mvg <- gamma g_mvg + (1 - gamma) g_cur
 *     g_est <- gamma g_mvg / (1 - gamma^t)
 * t >= 1 is the step counter after its increment.  The second line is kept as printed,
 * including its leading gamma (a factor common to all workers cancels in the weights);
 * 0 < gamma < 1 is required (gamma = 0 would make every estimate 0, gamma = 1 divides by 0). */
int oracle_norm_momentum(double *g_mvg, const double *g_cur, double *g_est, int64_t n,
                         double gamma, int64_t t)
{
    if (!g_mvg || !g_cur || !g_est || n < 0 || t < 1 || !(gamma > 0.0) || !(gamma < 1.0)) return 1;
    double denom = 1.0 - pow(gamma, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        g_mvg[i] = gamma * g_mvg[i] + (1.0 - gamma) * g_cur[i];
        g_est[i] = gamma * g_mvg[i] / denom;
    }
    return 0;
}

/* Model-level score from per-layer estimates under the MGRAWA policy (eq. (3) applied to the
 * estimates): A[m] = sum_k est[m][k]. */
int oracle_sum_layers(const double *est, int64_t K, int64_t L, double *A)
{
    if (!est || !A || K < 1 || L < 1) return 1;
    for (int64_t m = 0; m < K; ++m) {
        double a = 0.0;
        for (int64_t k = 0; k < L; ++k) a += est[m * L + k];
        A[m] = a;
    }
    return 0;
}

/* Local optimizer of the experiments (Appendix B.2.2: SGD, momentum, Nesterov acceleration,
 * weight decay), one step on a chunk.  The paper names the method but prints no formula; the
 * reading taken is the usual framework form of Nesterov's accelerated gradient,
 *     d   = grad + wd * x
 *     buf <- momentum * buf + d
 *     x   <- x - eta * (d + momentum * buf)
 * whose iterates are the look-ahead points x_t + momentum * v_t of the classical two-line form
 * v <- momentum v - eta grad(x + momentum v), x <- x + v  (a test checks that equivalence).
 * xd, buf: chunks [K][n] for columns i0..; g: the whole gradient array [K][ldg]. */
int oracle_nesterov_sgd(double *xd, double *buf, int64_t K, int64_t n, int64_t i0, const void *g,
                        int dtype, int64_t ldg, double eta, double momentum, double wd)
{
    if (!xd || !buf || !g || K < 1 || n < 0 || i0 < 0 || ldg < i0 + n) return 1;
    for (int64_t m = 0; m < K; ++m)
        for (int64_t i = 0; i < n; ++i) {
            double d = widen_at(g, dtype, m * ldg + i0 + i) + wd * xd[m * n + i];
            buf[m * n + i] = momentum * buf[m * n + i] + d;
            xd[m * n + i] = xd[m * n + i] - eta * (d + momentum * buf[m * n + i]);
        }
    return 0;
}

/* EASGD center (Appendix F, first algorithm), on a chunk: the workers' plain average x_a, then
 * the moving average in time  x_C <- (1 - rho) x_C + rho x_a.  The printed line reads
 * "(1 - rho) x_a + rho x_a", which is a no-op; the text (center = average of the workers "both
 * in space and time") fixes the reading with the previous center on the left. */
int oracle_easgd_center(const double *xd, int64_t K, int64_t n, double *c, double rho)
{
    if (!xd || !c || K < 1 || n < 0) return 1;
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t m = 0; m < K; ++m) s += xd[m * n + i];
        c[i] = (1.0 - rho) * c[i] + rho * (s / (double)K);
    }
    return 0;
}

/* LSGD leader (Appendix F, second algorithm): index of the worker with the smallest loss
 * (the first one on ties).  Returns -1 on a bad argument. */
int64_t oracle_leader(const double *loss, int64_t K)
{
    if (!loss || K < 1) return -1;
    int64_t best = 0;
    for (int64_t m = 1; m < K; ++m)
        if (loss[m] < loss[best]) best = m;
    return best;
}

/* Whether any of n scores is +inf, -inf or NaN (the paper leaves such scores undefined; the
 * update treats them by the weight formula and the library reports that it saw one). */
int oracle_nonfinite(const double *A, int64_t n)
{
    if (!A || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i)
        if (!isfinite(A[i])) return 1;
    return 0;
}
