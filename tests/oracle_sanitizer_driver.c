/*
 * Runs every function of the float64 CPU checker (oracle/grawa_oracle.c, compiled into this program
 * together with -fsanitize=address,undefined) once on a problem read from a file, with every buffer
 * allocated at exactly the size the function is entitled to touch, and writes all results to a second
 * file.  The test that builds this compares the results with those of the ordinary build of the same
 * source, so a read or write outside a buffer, a signed overflow or a misaligned access in the
 * checker's index arithmetic ends the run with a sanitizer report instead of going unnoticed.
 *
 * Input file: int64 K, L, ldx, ldg, dtype, i0, i1 ; double lambda, eta, mu, tau, gamma, momentum, wd, rho ;
 *             int64 off[L+1] ; float x[K*ldx] ; gradient bytes [K*ldg*(4|2)] ; double loss[K] ;
 *             double center_prev[i1-i0].
 * Output file: doubles, in the order of the calls below.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_sumsq(const void *, int, int64_t, int64_t, int64_t, const int64_t *, double *);
int oracle_layer_norms(const double *, int64_t, int64_t, double *);
int oracle_model_norms(const double *, int64_t, int64_t, int, double *);
int oracle_weights(const double *, int64_t, int64_t, double *);
int oracle_load_params(const float *, int64_t, int64_t, int64_t, int64_t, double *);
int oracle_local_sgd(double *, int64_t, int64_t, int64_t, const void *, int, int64_t, double);
int oracle_center(const double *, int64_t, int64_t, int64_t, const double *, int64_t, const int64_t *, double *);
int oracle_pull(double *, int64_t, int64_t, const double *, double);
int oracle_prox(double *, int64_t, int64_t, const double *, double, double);
int oracle_norm_momentum(double *, const double *, double *, int64_t, double, int64_t);
int oracle_sum_layers(const double *, int64_t, int64_t, double *);
int oracle_nesterov_sgd(double *, double *, int64_t, int64_t, int64_t, const void *, int, int64_t, double, double, double);
int oracle_easgd_center(const double *, int64_t, int64_t, double *, double);
int64_t oracle_leader(const double *, int64_t);

static void die(const char *what)
{
    fprintf(stderr, "oracle_sanitizer_driver: %s\n", what);
    exit(2);
}

static void *take(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || (bytes && fread(p, 1, bytes, f) != bytes)) die("short input");
    return p;
}

static double *fresh(size_t n)
{
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!p) die("out of memory");
    return p;
}

static void put(FILE *f, const double *p, size_t n)
{
    if (fwrite(p, sizeof(double), n, f) != n) die("short output");
}

#define OK(call) do { if ((call) != 0) die(#call " rejected its arguments"); } while (0)

int main(int argc, char **argv)
{
    if (argc != 3) die("usage: driver <input> <output>");
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) die("cannot open files");
    int64_t h[7];
    double s[8];
    if (fread(h, sizeof h, 1, in) != 1 || fread(s, sizeof s, 1, in) != 1) die("short header");
    const int64_t K = h[0], L = h[1], ldx = h[2], ldg = h[3], i0 = h[5], i1 = h[6], n = i1 - i0;
    const int dt = (int)h[4];
    const double lambda = s[0], eta = s[1], mu = s[2], tau = s[3], gamma = s[4], mom = s[5], wd = s[6], rho = s[7];
    int64_t *off = (int64_t *)take(in, sizeof(int64_t) * (size_t)(L + 1));
    float *x = (float *)take(in, sizeof(float) * (size_t)(K * ldx));
    void *g = take(in, (size_t)(K * ldg) * (dt == 1 ? 2 : 4));
    double *loss = (double *)take(in, sizeof(double) * (size_t)K);
    double *cprev = (double *)take(in, sizeof(double) * (size_t)n);
    const size_t KL = (size_t)(K * L), Kn = (size_t)(K * n);

    double *S = fresh(KL), *A = fresh(KL), *Am = fresh((size_t)K), *Af = fresh((size_t)K);
    double *bl = fresh(KL), *bm = fresh((size_t)K);
    OK(oracle_sumsq(g, dt, K, ldg, L, off, S));                 put(out, S, KL);
    OK(oracle_layer_norms(S, K, L, A));                         put(out, A, KL);
    OK(oracle_model_norms(S, K, L, 0, Am));                     put(out, Am, (size_t)K);
    OK(oracle_model_norms(S, K, L, 1, Af));                     put(out, Af, (size_t)K);
    OK(oracle_weights(A, K, L, bl));                            put(out, bl, KL);
    OK(oracle_weights(Am, K, 1, bm));                           put(out, bm, (size_t)K);

    double *xd = fresh(Kn), *c = fresh((size_t)n);
    OK(oracle_load_params(x, K, ldx, i0, i1, xd));
    OK(oracle_local_sgd(xd, K, n, i0, g, dt, ldg, eta));
    OK(oracle_prox(xd, K, n, cprev, mu, tau));
    OK(oracle_center(xd, K, n, i0, bl, L, off, c));
    OK(oracle_pull(xd, K, n, c, lambda));                       put(out, xd, Kn); put(out, c, (size_t)n);
    OK(oracle_load_params(x, K, ldx, i0, i1, xd));
    OK(oracle_center(xd, K, n, i0, bm, 1, NULL, c));
    OK(oracle_pull(xd, K, n, c, lambda));                       put(out, xd, Kn); put(out, c, (size_t)n);

    double *mvg = (double *)calloc(KL ? KL : 1, sizeof(double)), *est = fresh(KL), *sl = fresh((size_t)K);
    if (!mvg) die("out of memory");
    OK(oracle_norm_momentum(mvg, A, est, (int64_t)KL, gamma, 1));
    OK(oracle_norm_momentum(mvg, A, est, (int64_t)KL, gamma, 2)); put(out, mvg, KL); put(out, est, KL);
    OK(oracle_sum_layers(est, K, L, sl));                       put(out, sl, (size_t)K);

    double *buf = (double *)calloc(Kn ? Kn : 1, sizeof(double));
    if (!buf) die("out of memory");
    OK(oracle_load_params(x, K, ldx, i0, i1, xd));
    OK(oracle_nesterov_sgd(xd, buf, K, n, i0, g, dt, ldg, eta, mom, wd));
    OK(oracle_nesterov_sgd(xd, buf, K, n, i0, g, dt, ldg, eta, mom, wd)); put(out, xd, Kn); put(out, buf, Kn);

    OK(oracle_load_params(x, K, ldx, i0, i1, xd));
    memcpy(c, cprev, sizeof(double) * (size_t)n);
    OK(oracle_easgd_center(xd, K, n, c, rho));                  put(out, c, (size_t)n);
    const double lead = (double)oracle_leader(loss, K);         put(out, &lead, 1);

    free(off); free(x); free(g); free(loss); free(cprev); free(S); free(A); free(Am); free(Af); free(bl); free(bm);
    free(xd); free(c); free(mvg); free(est); free(sl); free(buf);
    if (fclose(out) != 0) die("close failed");
    fclose(in);
    return 0;
}
