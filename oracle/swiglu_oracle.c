/*
 * fp64 CPU oracle for the SwiGLU MLP block (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the checker, not the product: only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP library and is built with plain gcc.
 *
 * What it computes is the plain definition of the block (Background section,
 * the SwiGLU equations; Method section, the two-stage split):
 *
 *     A_gate = X W_gate            A_1 = X W_up
 *     A_silu = Sigmoid(A_gate) (x) A_gate          ((x) = elementwise)
 *     A_2    = A_1 (x) A_silu
 *     Y      = A_2 W_down
 *
 * with W_gate, W_up in R^{d_model x d_ff} and W_down in R^{d_ff x d_model}.
 * The method is exact (fusion moves intermediates, it does not change the
 * function), so the oracle is the definition written out: every input element
 * is widened exactly to fp64, every sum runs in ascending index order in
 * fp64, nothing is rounded on the way and the result is returned as fp64.
 *
 * Storage layouts (the paper gives only the mathematical shapes):
 *     X      row-major [M, d_model]
 *     W_gate row-major [d_ff, d_model]   (transposed mathematical shape)
 *     W_up   row-major [d_ff, d_model]   (transposed mathematical shape)
 *     W_down row-major [d_ff, d_model]   (the mathematical shape)
 *     Y      row-major [M, d_model], fp64
 * Element types: dtype 0 = bfloat16 bit patterns (uint16_t), 1 = IEEE fp32,
 * 2 = IEEE binary16 bit patterns (uint16_t).
 *
 * Threads only partition independent output elements (columns of d_ff in
 * stage one, columns of d_model in stage two); each output element is
 * produced by exactly one thread with a fixed summation order, so the result
 * does not depend on the thread count.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_BF16 0
#define ORACLE_FP32 1
#define ORACLE_FP16 2
#define ORACLE_FP64 3   /* internal: X already in fp64 (the normalised input of the decoder-layer form) */

/* Exact widening of one stored element to fp64. */
static double widen(const void *base, size_t idx, int dtype)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    if (dtype == ORACLE_FP16) {
        /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        uint16_t h = ((const uint16_t *)base)[idx];
        int sign = h >> 15, e = (h >> 10) & 31, frac = h & 1023;
        double v;
        if (e == 0) v = ldexp((double)frac, -24);                  /* zero and subnormals */
        else if (e == 31) v = frac ? NAN : INFINITY;
        else v = ldexp((double)(1024 + frac), e - 25);             /* (1 + frac/1024) * 2^(e-15) */
        return sign ? -v : v;
    }
    if (dtype == ORACLE_FP64) return ((const double *)base)[idx];
    return (double)((const float *)base)[idx];
}

/* SiLU(g) = Sigmoid(g) * g = g / (1 + exp(-g))   (Background, SwiGLU eq.). */
double oracle_silu(double g)
{
    return g / (1.0 + exp(-g));
}

typedef struct {
    const void *X, *Wg, *Wu, *Wd;
    double *G, *U, *A2, *Y;
    int M, d_model, d_ff, dtype;
    int xdtype; /* element type of X (= dtype, or ORACLE_FP64) */
    int lo, hi; /* this thread's range of columns */
} job_t;

/* Stage one, one thread's columns j in [lo, hi):
 *   G[m,j] = sum_k X[m,k] W_gate[k,j],  U[m,j] = sum_k X[m,k] W_up[k,j],
 *   A2[m,j] = U[m,j] * SiLU(G[m,j]). */
static void *stage_one(void *arg)
{
    job_t *t = (job_t *)arg;
    for (int j = t->lo; j < t->hi; ++j) {
        for (int m = 0; m < t->M; ++m) {
            double g = 0.0, u = 0.0;
            for (int k = 0; k < t->d_model; ++k) {
                double x = widen(t->X, (size_t)m * t->d_model + k, t->xdtype);
                g += x * widen(t->Wg, (size_t)j * t->d_model + k, t->dtype);
                u += x * widen(t->Wu, (size_t)j * t->d_model + k, t->dtype);
            }
            size_t o = (size_t)m * t->d_ff + j;
            if (t->G) t->G[o] = g;
            if (t->U) t->U[o] = u;
            t->A2[o] = u * oracle_silu(g);
        }
    }
    return NULL;
}

/* Stage two, one thread's columns n in [lo, hi):
 *   Y[m,n] = sum_j A2[m,j] W_down[j,n], j ascending. */
static void *stage_two(void *arg)
{
    job_t *t = (job_t *)arg;
    for (int m = 0; m < t->M; ++m) {
        double *y = t->Y + (size_t)m * t->d_model;
        for (int n = t->lo; n < t->hi; ++n) y[n] = 0.0;
        for (int j = 0; j < t->d_ff; ++j) {
            double a = t->A2[(size_t)m * t->d_ff + j];
            for (int n = t->lo; n < t->hi; ++n)
                y[n] += a * widen(t->Wd, (size_t)j * t->d_model + n, t->dtype);
        }
    }
    return NULL;
}

static int run_partitioned(void *(*fn)(void *), job_t *proto, int extent, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
    if (nthreads > extent) nthreads = extent > 0 ? extent : 1;
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    job_t *jobs = (job_t *)malloc(sizeof(job_t) * (size_t)nthreads);
    if (!th || !jobs) { free(th); free(jobs); return -2; }
    int started = 0;
    for (int i = 0; i < nthreads; ++i) {
        jobs[i] = *proto;
        jobs[i].lo = (int)((int64_t)extent * i / nthreads);
        jobs[i].hi = (int)((int64_t)extent * (i + 1) / nthreads);
        if (pthread_create(&th[i], NULL, fn, &jobs[i]) != 0) break;
        ++started;
    }
    for (int i = 0; i < started; ++i) pthread_join(th[i], NULL);
    int rc = (started == nthreads) ? 0 : -3;
    free(th); free(jobs);
    return rc;
}

/*
 * Stage one alone.  G, U may be NULL; A2 [M, d_ff] fp64 is required.
 * Returns 0, or a negative value on bad arguments / allocation failure.
 */
int oracle_gate_up_silu(const void *X, const void *Wg, const void *Wu,
                        double *G, double *U, double *A2,
                        int M, int d_model, int d_ff, int dtype, int nthreads)
{
    if (!X || !Wg || !Wu || !A2 || M < 1 || d_model < 1 || d_ff < 1) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32 && dtype != ORACLE_FP16) return -1;
    job_t p;
    memset(&p, 0, sizeof p);
    p.X = X; p.Wg = Wg; p.Wu = Wu; p.G = G; p.U = U; p.A2 = A2;
    p.M = M; p.d_model = d_model; p.d_ff = d_ff; p.dtype = dtype; p.xdtype = dtype;
    return run_partitioned(stage_one, &p, d_ff, nthreads);
}

/* Stage two alone: Y = A2 W_down, A2 given in fp64. */
int oracle_down(const double *A2, const void *Wd, double *Y,
                int M, int d_model, int d_ff, int dtype, int nthreads)
{
    if (!A2 || !Wd || !Y || M < 1 || d_model < 1 || d_ff < 1) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32 && dtype != ORACLE_FP16) return -1;
    job_t p;
    memset(&p, 0, sizeof p);
    p.A2 = (double *)A2; p.Wd = Wd; p.Y = Y;
    p.M = M; p.d_model = d_model; p.d_ff = d_ff; p.dtype = dtype;
    return run_partitioned(stage_two, &p, d_model, nthreads);
}

/* The whole block: Y = (SiLU(X W_gate) (x) (X W_up)) W_down, Y in fp64. */
int oracle_swiglu_mlp(const void *X, const void *Wg, const void *Wu, const void *Wd,
                      double *Y, int M, int d_model, int d_ff, int dtype, int nthreads)
{
    if (!Wd || !Y || M < 1 || d_ff < 1) return -1;
    double *A2 = (double *)malloc(sizeof(double) * (size_t)M * (size_t)d_ff);
    if (!A2) return -2;
    int rc = oracle_gate_up_silu(X, Wg, Wu, NULL, NULL, A2, M, d_model, d_ff, dtype, nthreads);
    if (rc == 0) rc = oracle_down(A2, Wd, Y, M, d_model, d_ff, dtype, nthreads);
    free(A2);
    return rc;
}

/*
 * Weighted RMS normalisation of every row, in fp64, nothing rounded:
 *   N[m,k] = H[m,k] * w[k] / sqrt( (1/d_model) sum_k H[m,k]^2 + eps ).
 * (The pre-normalisation of a decoder layer's MLP sub-block; not part of the
 * paper's block, which starts at X.  w == NULL means w = 1.)
 */
int oracle_rmsnorm(const void *H, const void *w, double *N, int M, int d_model, int dtype, double eps)
{
    if (!H || !N || M < 1 || d_model < 1) return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_FP32 && dtype != ORACLE_FP16) return -1;
    for (int m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int k = 0; k < d_model; ++k) {
            double h = widen(H, (size_t)m * d_model + k, dtype);
            ss += h * h;
        }
        double r = sqrt(ss / (double)d_model + eps);
        for (int k = 0; k < d_model; ++k) {
            double h = widen(H, (size_t)m * d_model + k, dtype);
            double wk = w ? widen(w, (size_t)k, dtype) : 1.0;
            N[(size_t)m * d_model + k] = h * wk / r;
        }
    }
    return 0;
}

/*
 * The MLP sub-block of a pre-norm decoder layer around the paper's block:
 *   H_out = H + SwiGLU_MLP( RMSNorm(H; w, eps) ),   H_out in fp64.
 */
int oracle_mlp_block(const void *H, const void *w, double eps,
                     const void *Wg, const void *Wu, const void *Wd,
                     double *Y, int M, int d_model, int d_ff, int dtype, int nthreads)
{
    if (!H || !Wg || !Wu || !Wd || !Y || M < 1 || d_model < 1 || d_ff < 1) return -1;
    double *N = (double *)malloc(sizeof(double) * (size_t)M * (size_t)d_model);
    double *A2 = (double *)malloc(sizeof(double) * (size_t)M * (size_t)d_ff);
    if (!N || !A2) { free(N); free(A2); return -2; }
    int rc = oracle_rmsnorm(H, w, N, M, d_model, dtype, eps);
    if (rc == 0) {
        job_t p;
        memset(&p, 0, sizeof p);
        p.X = N; p.Wg = Wg; p.Wu = Wu; p.A2 = A2;
        p.M = M; p.d_model = d_model; p.d_ff = d_ff; p.dtype = dtype; p.xdtype = ORACLE_FP64;
        rc = run_partitioned(stage_one, &p, d_ff, nthreads);
    }
    if (rc == 0) rc = oracle_down(A2, Wd, Y, M, d_model, d_ff, dtype, nthreads);
    if (rc == 0)
        for (size_t i = 0; i < (size_t)M * (size_t)d_model; ++i) Y[i] += widen(H, i, dtype);
    free(N); free(A2);
    return rc;
}
