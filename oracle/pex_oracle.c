/*
 * pex_oracle.c -- fp64 CPU oracle for the per-example gradient statistics of a
 * dense layer in a sequence model.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP library and is never a fallback for it.
 *
 * What it is: the "memory intensive" route of Sec. 2.1 written out for one dense
 * sequence layer (Sec. 2.3, "Dense layers in sequence-level architectures"):
 * materialise every per-example weight gradient M_b = X_b^T G_b, apply phi
 * element by element, and sum over the batch.  No blocking, no fusion, no
 * reordering beyond that definition.  Inputs are float arrays holding the
 * already-rounded bf16 (or fp32) payloads; every product and sum is fp64.
 *
 * Notation (paper -> here): H -> X[B,T,din], Lambda -> G[B,T,dout], L -> T,
 * D -> din, F -> dout, M -> M_b, S -> S_*, S' -> S_tok.
 *
 * Pins (tests/test_oracle_pins.py): worked all-ones example of App. A, the
 * batch-gradient identity, T=1 factorisation for square and sign (Sec. 2.3,
 * MLP paragraph), B=1 reductions, ghost-norm Gram-matrix route, Cauchy-Schwarz
 * ordering of nu_micro and nu_adam (Sec. 3.2), scaling/sign-flip/permutation
 * laws, library einsum on small shapes, long-double brute force.
 *
 * OpenMP parallelises over output rows i only (each thread owns whole rows of
 * M_b / S, so there is no reduction-order ambiguity between threads).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PEX_ORACLE_OK 0
#define PEX_ORACLE_BAD_ARG 1
#define PEX_ORACLE_NOMEM 2

/* relative width of the sign-ambiguity band, per example, relative to max|M_b| */
#define PEX_ORACLE_SIGN_BAND 1e-6

int pex_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * One per-example gradient, materialised (Sec. 2.3: M = einsum(BLD,BLF->BDF),
 * here for a single b):  M[i][j] = sum_t X[b,t,i] * G[b,t,j].
 */
static void per_example_gradient(const float *Xb, const float *Gb, int64_t T, int64_t din,
                                 int64_t dout, double *M)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < din; ++i) {
        double *Mi = M + i * dout;
        for (int64_t j = 0; j < dout; ++j) Mi[j] = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            const double x = (double)Xb[t * din + i];
            const float *g = Gb + t * dout;
            for (int64_t j = 0; j < dout; ++j) Mi[j] += x * (double)g[j];
        }
    }
}

/*
 * S_id  = sum_b M_b            (the ordinary batch weight gradient)
 * S_sq  = sum_b M_b o M_b      (Sec. 2.3: S = sum over b of M squared; B * nu_micro of Eq. nu_defs)
 * S_sgn = sum_b sgn(M_b)       (Sec. 3.1: avg o sign, before the 1/B; sgn(0) = 0)
 * amb[i][j]  = number of examples b with |M_b[i][j]| < 1e-6 * max_ij |M_b|  (sign-ambiguity count)
 * maxabs[b]  = max_ij |M_b[i][j]|
 * normsq[b]  = ||M_b||_F^2     (the per-example squared norm of the ghost-norm remark, Sec. 2.3)
 * Any output pointer may be NULL.  Outputs are overwritten.
 */
int pex_oracle_stat(const float *X, const float *G, int64_t B, int64_t T, int64_t din,
                    int64_t dout, double *S_id, double *S_sq, double *S_sgn, int32_t *amb,
                    double *maxabs, double *normsq)
{
    if (!X || !G || B < 1 || T < 1 || din < 1 || dout < 1) return PEX_ORACLE_BAD_ARG;
    const int64_t n = din * dout;
    double *M = (double *)malloc((size_t)n * sizeof(double));
    if (!M) return PEX_ORACLE_NOMEM;
    if (S_id) memset(S_id, 0, (size_t)n * sizeof(double));
    if (S_sq) memset(S_sq, 0, (size_t)n * sizeof(double));
    if (S_sgn) memset(S_sgn, 0, (size_t)n * sizeof(double));
    if (amb) memset(amb, 0, (size_t)n * sizeof(int32_t));

    for (int64_t b = 0; b < B; ++b) {
        per_example_gradient(X + b * T * din, G + b * T * dout, T, din, dout, M);

        double mx = 0.0;
#pragma omp parallel for schedule(static) reduction(max : mx)
        for (int64_t e = 0; e < n; ++e) {
            const double a = fabs(M[e]);
            if (a > mx) mx = a;
        }
        if (maxabs) maxabs[b] = mx;
        const double band = PEX_ORACLE_SIGN_BAND * mx;

        double nsq = 0.0;
        for (int64_t e = 0; e < n; ++e) nsq += M[e] * M[e];
        if (normsq) normsq[b] = nsq;

#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            const double m = M[e];
            if (S_id) S_id[e] += m;
            if (S_sq) S_sq[e] += m * m;
            if (S_sgn) S_sgn[e] += (double)((m > 0.0) - (m < 0.0));
            if (amb) amb[e] += (fabs(m) < band) ? 1 : 0;
        }
    }
    free(M);
    return PEX_ORACLE_OK;
}

/*
 * Per-example gradients at n sampled output positions (ii[k], jj[k]) only:
 * Mout[b*n + k] = sum_t X[b,t,ii[k]] * G[b,t,jj[k]].  Same definition as above,
 * evaluated entry by entry, for sizes where the full din x dout matrix is too
 * slow to materialise on the CPU.  The caller applies phi and sums over b.
 */
int pex_oracle_per_example_at(const float *X, const float *G, int64_t B, int64_t T, int64_t din,
                              int64_t dout, int64_t n, const int64_t *ii, const int64_t *jj,
                              double *Mout)
{
    if (!X || !G || !ii || !jj || !Mout || B < 1 || T < 1 || din < 1 || dout < 1 || n < 0)
        return PEX_ORACLE_BAD_ARG;
    for (int64_t k = 0; k < n; ++k)
        if (ii[k] < 0 || ii[k] >= din || jj[k] < 0 || jj[k] >= dout) return PEX_ORACLE_BAD_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t k = 0; k < n; ++k) {
            const float *x = X + b * T * din + ii[k];
            const float *g = G + b * T * dout + jj[k];
            double s = 0.0;
            for (int64_t t = 0; t < T; ++t) s += (double)x[t * din] * (double)g[t * dout];
            Mout[b * n + k] = s;
        }
    }
    return PEX_ORACLE_OK;
}

/*
 * Per-token square statistic (Sec. 2.3, "per-token second moments"):
 * S_tok[i][j] = sum_b sum_t X[b,t,i]^2 * G[b,t,j]^2.
 */
int pex_oracle_token_sq(const float *X, const float *G, int64_t B, int64_t T, int64_t din,
                        int64_t dout, double *S_tok)
{
    if (!X || !G || !S_tok || B < 1 || T < 1 || din < 1 || dout < 1) return PEX_ORACLE_BAD_ARG;
    const int64_t BT = B * T;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < din; ++i) {
        double *Si = S_tok + i * dout;
        for (int64_t j = 0; j < dout; ++j) Si[j] = 0.0;
        for (int64_t r = 0; r < BT; ++r) {
            const double x = (double)X[r * din + i];
            const double x2 = x * x;
            const float *g = G + r * dout;
            for (int64_t j = 0; j < dout; ++j) {
                const double gv = (double)g[j];
                Si[j] += x2 * (gv * gv);
            }
        }
    }
    return PEX_ORACLE_OK;
}

/* Per-token square at sampled positions: out[k] = sum_{b,t} X[b,t,ii[k]]^2 G[b,t,jj[k]]^2. */
int pex_oracle_token_sq_at(const float *X, const float *G, int64_t B, int64_t T, int64_t din,
                           int64_t dout, int64_t n, const int64_t *ii, const int64_t *jj,
                           double *out)
{
    if (!X || !G || !ii || !jj || !out || B < 1 || T < 1 || din < 1 || dout < 1 || n < 0)
        return PEX_ORACLE_BAD_ARG;
    for (int64_t k = 0; k < n; ++k)
        if (ii[k] < 0 || ii[k] >= din || jj[k] < 0 || jj[k] >= dout) return PEX_ORACLE_BAD_ARG;
    const int64_t BT = B * T;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        const float *x = X + ii[k];
        const float *g = G + jj[k];
        double s = 0.0;
        for (int64_t r = 0; r < BT; ++r) {
            const double xv = (double)x[r * din], gv = (double)g[r * dout];
            s += (xv * xv) * (gv * gv);
        }
        out[k] = s;
    }
    return PEX_ORACLE_OK;
}
