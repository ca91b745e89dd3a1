/*
 * came_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, double-precision CPU transcription of one CAME optimizer
 * step (Luo et al., "CAME: Confidence-guided Adaptive Memory Efficient
 * Optimization", Algorithm 2) and of the Adafactor-with-momentum step it
 * extends (Algorithm 1).  It exists only so that tests, the smoke check and
 * the benchmark's cpu_baseline leg have something independent to compare the
 * GPU library against.  It shares no code, header, table or helper with the
 * HIP path and must never be linked into or called from it.
 *
 * Conventions (Section 3.1): a weight matrix theta is n x m, row-major,
 * n = rows, m = columns.  1_m is a column of m ones, so "(X) 1_m" is the
 * vector of row sums (length n) and "1_n^T (X)" the vector of column sums
 * (length m).  All reductions are SUMS, as printed -- not means.
 *
 * Every intermediate of Algorithm 2 (g^2+eps1, v, u, u_hat, U, S) is
 * materialised as a dense n x m array, in the paper's notation, and each step
 * of the algorithm is one plain loop over it, in the algorithm's order
 * (second-moment statistics, rank-one second moment, raw and clipped update,
 * momentum, instability, confidence statistics, rank-one instability, step),
 * so the code can be checked against the paper by eye.  No blocking, fusion or
 * algebraic rewriting.
 *
 * Readings where the paper is silent (all listed in the design document):
 *   - R_0 = C_0 = 0, like r_0, c_0, m_0 (Algorithm 2's input list names only
 *     the latter three).
 *   - no bias correction and constant beta's: the step counter t never enters
 *     the arithmetic of Algorithm 2.
 *   - RMS(u_t) is over the n*m components of this tensor's u_t (text below
 *     Eq. 1).
 *   - U_t uses the NEW momentum m_t (Algorithm 2, instability line).
 *   - 1-D parameters: Algorithm 2 applied to an n x 1 matrix.  There
 *     c_t = 1^T r_t, hence v_t = r_t and S_t = R_t: the unfactored update.
 *     came_oracle_vector_step writes that special case out; a test pins it to
 *     came_oracle_matrix_step on shape n x 1.
 *
 *   - reduced-precision momentum (not in the paper): see came_oracle_round_bf16.
 *
 * Pinned by tests/test_oracle_pins.py (closed forms, invariants, dense brute
 * force, a hand-checkable worked example, mutation checks).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    double beta1, beta2, beta3; /* EMA coefficients of m, (r,c), (R,C) */
    double eps1, eps2;          /* regularisation constants            */
    double clip_d;              /* clipping threshold d of Eq. 1       */
    double lr;                  /* learning rate eta                   */
} came_oracle_hyper;

/* diag[0] = RMS(u_t), diag[1] = RMS(u_hat_t); diag may be NULL. */

static double rms_of(const double *x, int64_t count)
{
    /* root-mean-square of the components (text below Eq. 1) */
    double ss = 0.0;
    for (int64_t k = 0; k < count; ++k) ss += x[k] * x[k];
    return sqrt(ss / (double)count);
}

/*
 * One step of Algorithm 2 on one n x m matrix.
 * theta, g, M: n*m doubles (row-major).  r, R: n doubles.  c, C: m doubles.
 * theta, M, r, c, R, C are updated in place.  Returns 0, or -1 on allocation
 * failure / bad sizes.
 */
int came_oracle_matrix_step(int64_t n, int64_t m, double *theta, const double *g,
                            double *M, double *r, double *c, double *R, double *C,
                            const came_oracle_hyper *h, double *diag)
{
    if (n <= 0 || m <= 0) return -1;
    const int64_t nm = n * m;
    double *G = malloc(sizeof(double) * nm);    /* g^2 + eps1 1_n 1_m^T */
    double *v = malloc(sizeof(double) * nm);    /* v_t                  */
    double *u = malloc(sizeof(double) * nm);    /* u_t                  */
    double *uh = malloc(sizeof(double) * nm);   /* u_hat_t              */
    double *U = malloc(sizeof(double) * nm);    /* instability U_t      */
    double *S = malloc(sizeof(double) * nm);    /* S_t                  */
    if (!G || !v || !u || !uh || !U || !S) {
        free(G); free(v); free(u); free(uh); free(U); free(S);
        return -1;
    }

    /* the regularised squared gradient, entry by entry */
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            G[i * m + j] = g[i * m + j] * g[i * m + j] + h->eps1;

    /* second-moment row statistic: moving average (beta2) of the ROW SUMS of G */
    for (int64_t i = 0; i < n; ++i) {
        double rowsum = 0.0;
        for (int64_t j = 0; j < m; ++j) rowsum += G[i * m + j];
        r[i] = h->beta2 * r[i] + (1.0 - h->beta2) * rowsum;
    }
    /* second-moment column statistic: moving average (beta2) of the COLUMN SUMS of G */
    for (int64_t j = 0; j < m; ++j) {
        double colsum = 0.0;
        for (int64_t i = 0; i < n; ++i) colsum += G[i * m + j];
        c[j] = h->beta2 * c[j] + (1.0 - h->beta2) * colsum;
    }

    /* rank-one second moment: outer product of the two statistics over the total of r */
    double sum_r = 0.0;
    for (int64_t i = 0; i < n; ++i) sum_r += r[i];
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            v[i * m + j] = r[i] * c[j] / sum_r;

    /* the raw update: gradient over the root of the second moment */
    for (int64_t k = 0; k < nm; ++k) u[k] = g[k] / sqrt(v[k]);

    /* clipping (Eq. 1): scaled down, never up, so that its RMS does not exceed d */
    const double rms_u = rms_of(u, nm);
    const double denom = fmax(1.0, rms_u / h->clip_d);
    for (int64_t k = 0; k < nm; ++k) uh[k] = u[k] / denom;

    /* momentum: moving average (beta1) of the clipped update */
    for (int64_t k = 0; k < nm; ++k) M[k] = h->beta1 * M[k] + (1.0 - h->beta1) * uh[k];

    /* instability: squared distance between the clipped update and the NEW momentum */
    for (int64_t k = 0; k < nm; ++k) U[k] = (uh[k] - M[k]) * (uh[k] - M[k]);

    /* confidence row statistic: moving average (beta3) of the row sums of U + eps2 */
    for (int64_t i = 0; i < n; ++i) {
        double rowsum = 0.0;
        for (int64_t j = 0; j < m; ++j) rowsum += U[i * m + j] + h->eps2;
        R[i] = h->beta3 * R[i] + (1.0 - h->beta3) * rowsum;
    }
    /* confidence column statistic: the same over the columns */
    for (int64_t j = 0; j < m; ++j) {
        double colsum = 0.0;
        for (int64_t i = 0; i < n; ++i) colsum += U[i * m + j] + h->eps2;
        C[j] = h->beta3 * C[j] + (1.0 - h->beta3) * colsum;
    }

    /* rank-one instability estimate, formed from R and C the way v is formed from r and c */
    double sum_R = 0.0;
    for (int64_t i = 0; i < n; ++i) sum_R += R[i];
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            S[i * m + j] = R[i] * C[j] / sum_R;

    /* the step: the momentum over the root of the instability estimate, times the learning rate */
    for (int64_t k = 0; k < nm; ++k) theta[k] = theta[k] - h->lr / sqrt(S[k]) * M[k];

    if (diag) { diag[0] = rms_u; diag[1] = rms_of(uh, nm); }
    free(G); free(v); free(u); free(uh); free(U); free(S);
    return 0;
}

/*
 * Algorithm 2 on a 1-D parameter of length n, i.e. the n x 1 special case
 * written out: the second moment v (length n) and the confidence s (length n)
 * are kept unfactored.  theta, M, v, s updated in place.
 */
int came_oracle_vector_step(int64_t n, double *theta, const double *g, double *M,
                            double *v, double *s, const came_oracle_hyper *h, double *diag)
{
    if (n <= 0) return -1;
    double *u = malloc(sizeof(double) * n);
    double *uh = malloc(sizeof(double) * n);
    if (!u || !uh) { free(u); free(uh); return -1; }

    /* unfactored second moment and raw update */
    for (int64_t i = 0; i < n; ++i) {
        v[i] = h->beta2 * v[i] + (1.0 - h->beta2) * (g[i] * g[i] + h->eps1);
        u[i] = g[i] / sqrt(v[i]);
    }
    /* Eq. 1 over the n components */
    const double rms_u = rms_of(u, n);
    const double denom = fmax(1.0, rms_u / h->clip_d);
    for (int64_t i = 0; i < n; ++i) uh[i] = u[i] / denom;
    /* momentum, instability, unfactored confidence, update */
    for (int64_t i = 0; i < n; ++i) {
        M[i] = h->beta1 * M[i] + (1.0 - h->beta1) * uh[i];
        const double U = (uh[i] - M[i]) * (uh[i] - M[i]);
        s[i] = h->beta3 * s[i] + (1.0 - h->beta3) * (U + h->eps2);
        theta[i] = theta[i] - h->lr / sqrt(s[i]) * M[i];
    }
    if (diag) { diag[0] = rms_u; diag[1] = rms_of(uh, n); }
    free(u); free(uh);
    return 0;
}

/*
 * Dense brute force, O(nm) state: keeps the FULL second-moment EMA
 *   V_t = beta2 V_{t-1} + (1-beta2)(g^2 + eps1)
 * and the FULL instability EMA
 *   Ubar_t = beta3 Ubar_{t-1} + (1-beta3)(U_t + eps2),
 * and factors each with the rank-1 solution of Eq. 2,
 *   W = X 1_m,   H = 1_n^T X / (1_n^T X 1_m),   X ~ W H,
 * every step.  By linearity of the EMAs the factored quantities of
 * Algorithm 2 are r = V 1_m, c = 1_n^T V, R = Ubar 1_m, C = 1_n^T Ubar; they
 * are written to r_out, c_out, R_out, C_out for comparison.  This is the
 * memory-hungry method the factored one must reproduce (Section 3.1, last
 * paragraph; Section 3.3, paragraph on factorising U_t).
 */
int came_oracle_dense_step(int64_t n, int64_t m, double *theta, const double *g,
                           double *M, double *V, double *Ubar,
                           double *r_out, double *c_out, double *R_out, double *C_out,
                           const came_oracle_hyper *h)
{
    if (n <= 0 || m <= 0) return -1;
    const int64_t nm = n * m;
    double *W = malloc(sizeof(double) * n);
    double *H = malloc(sizeof(double) * m);
    double *uh = malloc(sizeof(double) * nm);
    if (!W || !H || !uh) { free(W); free(H); free(uh); return -1; }

    for (int64_t k = 0; k < nm; ++k)
        V[k] = h->beta2 * V[k] + (1.0 - h->beta2) * (g[k] * g[k] + h->eps1);

    /* Eq. 2 on V */
    double total = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        W[i] = 0.0;
        for (int64_t j = 0; j < m; ++j) W[i] += V[i * m + j];
        total += W[i];
    }
    for (int64_t j = 0; j < m; ++j) {
        double colsum = 0.0;
        for (int64_t i = 0; i < n; ++i) colsum += V[i * m + j];
        c_out[j] = colsum;
        H[j] = colsum / total;
    }
    for (int64_t i = 0; i < n; ++i) r_out[i] = W[i];

    /* u = g / sqrt(W H), then Eq. 1 */
    double ss = 0.0;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j) {
            const double uij = g[i * m + j] / sqrt(W[i] * H[j]);
            uh[i * m + j] = uij;
            ss += uij * uij;
        }
    const double denom = fmax(1.0, sqrt(ss / (double)nm) / h->clip_d);
    for (int64_t k = 0; k < nm; ++k) uh[k] /= denom;

    for (int64_t k = 0; k < nm; ++k) {
        M[k] = h->beta1 * M[k] + (1.0 - h->beta1) * uh[k];
        const double U = (uh[k] - M[k]) * (uh[k] - M[k]);
        Ubar[k] = h->beta3 * Ubar[k] + (1.0 - h->beta3) * (U + h->eps2);
    }

    /* Eq. 2 on Ubar */
    total = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        W[i] = 0.0;
        for (int64_t j = 0; j < m; ++j) W[i] += Ubar[i * m + j];
        total += W[i];
    }
    for (int64_t j = 0; j < m; ++j) {
        double colsum = 0.0;
        for (int64_t i = 0; i < n; ++i) colsum += Ubar[i * m + j];
        C_out[j] = colsum;
        H[j] = colsum / total;
    }
    for (int64_t i = 0; i < n; ++i) R_out[i] = W[i];

    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            theta[i * m + j] -= h->lr * M[i * m + j] / sqrt(W[i] * H[j]);

    free(W); free(H); free(uh);
    return 0;
}

/*
 * One step of Algorithm 1 (Adafactor with momentum) on one n x m matrix:
 * Algorithm 2 without the instability/confidence lines; the parameter moves
 * by -eta m_t.
 */
int adafactor_oracle_matrix_step(int64_t n, int64_t m, double *theta, const double *g,
                                 double *M, double *r, double *c,
                                 const came_oracle_hyper *h, double *diag)
{
    if (n <= 0 || m <= 0) return -1;
    const int64_t nm = n * m;
    double *u = malloc(sizeof(double) * nm);
    if (!u) return -1;

    for (int64_t i = 0; i < n; ++i) {
        double rowsum = 0.0;
        for (int64_t j = 0; j < m; ++j) rowsum += g[i * m + j] * g[i * m + j] + h->eps1;
        r[i] = h->beta2 * r[i] + (1.0 - h->beta2) * rowsum;
    }
    for (int64_t j = 0; j < m; ++j) {
        double colsum = 0.0;
        for (int64_t i = 0; i < n; ++i) colsum += g[i * m + j] * g[i * m + j] + h->eps1;
        c[j] = h->beta2 * c[j] + (1.0 - h->beta2) * colsum;
    }
    double sum_r = 0.0;
    for (int64_t i = 0; i < n; ++i) sum_r += r[i];
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            u[i * m + j] = g[i * m + j] / sqrt(r[i] * c[j] / sum_r);
    const double rms_u = rms_of(u, nm);
    const double denom = fmax(1.0, rms_u / h->clip_d);
    for (int64_t k = 0; k < nm; ++k) {
        u[k] /= denom;
        M[k] = h->beta1 * M[k] + (1.0 - h->beta1) * u[k];
        theta[k] = theta[k] - h->lr * M[k];
    }
    if (diag) { diag[0] = rms_u; diag[1] = rms_of(u, nm); }
    free(u);
    return 0;
}

/*
 * Storage rounding of the reduced-precision-momentum variant (NOT in the paper, which
 * does not say in what precision the states are kept): the momentum is held in
 * bfloat16 between steps.  A step reads the stored value as m_{t-1}, forms m_t, U_t and
 * theta_t exactly as Algorithm 2 prints them, and only then replaces m_t by the nearest
 * bfloat16 for storage.  The GPU path takes that rounding decision on a binary32 m_t,
 * so the value is first rounded to binary32 here as well.
 *
 * bfloat16 is binary32 cut to its upper 16 bits: 1 sign, 8 exponent, 7 fraction bits,
 * i.e. 8 significant bits over binary32's exponent range; its subnormals are the
 * multiples of 2^-133.  Rounding is to nearest, ties to the even significand.
 */
double came_oracle_round_bf16(double x)
{
    if (isnan(x) || isinf(x) || x == 0.0) return x;
    const double f = (double)(float)x;           /* the binary32 the kernel would hold */
    if (isinf(f) || f == 0.0) return f;
    int e;
    (void)frexp(f, &e);                          /* |f| = mant * 2^e with mant in [0.5, 1) */
    int q = e - 8;                               /* 8 significant bits: spacing 2^(e-8) */
    if (q < -133) q = -133;                      /* never finer than the subnormal spacing */
    const double steps = nearbyint(ldexp(f, -q)); /* default rounding mode: ties to even */
    const double y = ldexp(steps, q);
    if (fabs(y) >= ldexp(1.0, 128)) return copysign(INFINITY, y);
    return y;
}

/* came_oracle_round_bf16 applied to every element of x, in place. */
void came_oracle_store_bf16(double *x, int64_t count)
{
    for (int64_t k = 0; k < count; ++k) x[k] = came_oracle_round_bf16(x[k]);
}

/*
 * Decoupled weight decay (NOT in the paper; the usual companion of such optimizers in
 * practice): before the step's update the parameter shrinks by eta * lambda * theta,
 *   theta <- theta - eta lambda theta,
 * independently of the gradient statistics.  The step functions above then run unchanged
 * on the shrunk theta.
 */
void came_oracle_decay(double *theta, int64_t count, double lr, double weight_decay)
{
    for (int64_t k = 0; k < count; ++k) theta[k] = theta[k] - lr * weight_decay * theta[k];
}

/*
 * One CAME step over a list of tensors.  Tensors are independent (Algorithm 2
 * is stated per parameter matrix), so the only parallelism is one tensor per
 * OpenMP thread; the arithmetic of each tensor is the serial code above.
 * ndim[t] == 2: matrix rows[t] x cols[t] with state M,r,c,R,C.
 * ndim[t] == 1: vector of rows[t] entries with state M, r(=v), R(=s);
 *               c[t], C[t] are ignored.
 * nthreads <= 0: leave the OpenMP default.  Returns 0 or the first failure.
 */
int came_oracle_step_list(int32_t ntensors, const int64_t *rows, const int64_t *cols,
                          const int32_t *ndim, double *const *theta, const double *const *g,
                          double *const *M, double *const *r, double *const *c,
                          double *const *R, double *const *C,
                          const came_oracle_hyper *h, int32_t nthreads)
{
    int rc = 0;
    int nt = 1;
    (void)nt;
    (void)nthreads;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    nt = nthreads > 0 ? nthreads : omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nt)
#endif
    for (int32_t t = 0; t < ntensors; ++t) {
        int e;
        if (ndim[t] == 2)
            e = came_oracle_matrix_step(rows[t], cols[t], theta[t], g[t], M[t], r[t], c[t],
                                        R[t], C[t], h, NULL);
        else
            e = came_oracle_vector_step(rows[t], theta[t], g[t], M[t], r[t], R[t], h, NULL);
        if (e != 0) {
#ifdef _OPENMP
#pragma omp critical
#endif
            rc = e;
        }
    }
    return rc;
}

/* number of OpenMP threads a parallel region would get by default (1 without OpenMP) */
int32_t came_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
