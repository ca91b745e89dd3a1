/*
 * Driver for the CPU oracle, built together with oracle/came_oracle.c under
 * -fsanitize=address,undefined by tests/test_sanitizers.py.  Every array the oracle is handed
 * is an exact-size heap block, so an access one element past any of them is reported.  Runs a
 * few steps of every oracle routine on the shapes the pins use (1x1, n x 1, 1 x n, ragged
 * small matrices, vectors) and prints a checksum.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct { double beta1, beta2, beta3, eps1, eps2, clip_d, lr; } came_oracle_hyper;

int came_oracle_matrix_step(int64_t, int64_t, double *, const double *, double *, double *, double *, double *, double *,
                            const came_oracle_hyper *, double *);
int came_oracle_vector_step(int64_t, double *, const double *, double *, double *, double *, const came_oracle_hyper *, double *);
int came_oracle_dense_step(int64_t, int64_t, double *, const double *, double *, double *, double *, double *, double *,
                           double *, double *, const came_oracle_hyper *);
int adafactor_oracle_matrix_step(int64_t, int64_t, double *, const double *, double *, double *, double *,
                                 const came_oracle_hyper *, double *);
double came_oracle_round_bf16(double);
void came_oracle_store_bf16(double *, int64_t);
void came_oracle_decay(double *, int64_t, double, double);
int came_oracle_step_list(int32_t, const int64_t *, const int64_t *, const int32_t *, double *const *, const double *const *,
                          double *const *, double *const *, double *const *, double *const *, double *const *,
                          const came_oracle_hyper *, int32_t);

static uint64_t rng = 88172645463325252ull;
static double draw(void)
{
    rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
    return ((double)(rng >> 11) / 9007199254740992.0 - 0.5) * 0.2;
}
static double *block(int64_t count, int random)
{
    double *p = malloc(sizeof(double) * (size_t)count);
    if (!p) exit(4);
    for (int64_t k = 0; k < count; ++k) p[k] = random ? draw() : 0.0;
    return p;
}

int main(void)
{
    const came_oracle_hyper h = {0.9, 0.999, 0.9999, 1e-30, 1e-16, 1.0, 2e-4};
    const int64_t shapes[][2] = {{1, 1}, {1, 8}, {8, 1}, {3, 5}, {2, 3}, {7, 13}, {33, 17}};
    double sum = 0.0;
    for (size_t s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s) {
        const int64_t n = shapes[s][0], m = shapes[s][1], nm = n * m;
        double *th = block(nm, 1), *M = block(nm, 0), *r = block(n, 0), *c = block(m, 0), *R = block(n, 0), *C = block(m, 0);
        double *th2 = block(nm, 1), *M2 = block(nm, 0), *V = block(nm, 0), *Ub = block(nm, 0);
        double *ro = block(n, 0), *co = block(m, 0), *Ro = block(n, 0), *Co = block(m, 0);
        double *th3 = block(nm, 1), *M3 = block(nm, 0), *r3 = block(n, 0), *c3 = block(m, 0);
        double diag[2];
        for (int t = 0; t < 3; ++t) {
            double *g = block(nm, 1);
            if (t == 2) for (int64_t j = 0; j < m; ++j) g[j] = 0.0; /* an all-zero row: only eps1 is left */
            if (came_oracle_matrix_step(n, m, th, g, M, r, c, R, C, &h, diag)) return 5;
            if (came_oracle_dense_step(n, m, th2, g, M2, V, Ub, ro, co, Ro, Co, &h)) return 5;
            if (adafactor_oracle_matrix_step(n, m, th3, g, M3, r3, c3, &h, diag)) return 5;
            came_oracle_store_bf16(M, nm);
            came_oracle_decay(th, nm, h.lr, 0.1);
            free(g);
        }
        for (int64_t k = 0; k < nm; ++k) sum += th[k] + th2[k] + th3[k];
        free(th); free(M); free(r); free(c); free(R); free(C); free(th2); free(M2); free(V); free(Ub);
        free(ro); free(co); free(Ro); free(Co); free(th3); free(M3); free(r3); free(c3);
    }
    const int64_t lens[] = {1, 7, 256, 1001};
    for (size_t s = 0; s < sizeof(lens) / sizeof(lens[0]); ++s) {
        const int64_t n = lens[s];
        double *th = block(n, 1), *M = block(n, 0), *v = block(n, 0), *sv = block(n, 0);
        for (int t = 0; t < 3; ++t) {
            double *g = block(n, 1);
            if (came_oracle_vector_step(n, th, g, M, v, sv, &h, NULL)) return 5;
            free(g);
        }
        for (int64_t k = 0; k < n; ++k) sum += th[k];
        free(th); free(M); free(v); free(sv);
    }
    {   /* the list driver: one matrix, one vector */
        const int64_t rows[2] = {5, 9}, cols[2] = {6, 1};
        const int32_t ndim[2] = {2, 1};
        double *th[2] = {block(30, 1), block(9, 1)}, *M[2] = {block(30, 0), block(9, 0)};
        double *r[2] = {block(5, 0), block(9, 0)}, *c[2] = {block(6, 0), NULL};
        double *R[2] = {block(5, 0), block(9, 0)}, *C[2] = {block(6, 0), NULL};
        double *g[2] = {block(30, 1), block(9, 1)};
        const double *gc[2] = {g[0], g[1]};
        if (came_oracle_step_list(2, rows, cols, ndim, th, gc, M, r, c, R, C, &h, 2)) return 5;
        sum += th[0][29] + th[1][8];
        for (int k = 0; k < 2; ++k) { free(th[k]); free(M[k]); free(r[k]); free(c[k]); free(R[k]); free(C[k]); free(g[k]); }
    }
    sum += came_oracle_round_bf16(1.00390625) + came_oracle_round_bf16(-3.0e38) + came_oracle_round_bf16(1e-40);
    printf("checksum %.17g\n", sum);
    return 0;
}
