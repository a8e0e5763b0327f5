/*
 * Sanitizer driver for the CPU oracle: calls every exported routine of oracle/tsr_oracle.c on
 * small ragged shapes with exactly-sized heap buffers, so that an out-of-bounds index, a use of
 * uninitialised heap or an undefined operation inside the oracle's loops trips
 * AddressSanitizer / UndefinedBehaviorSanitizer.  Built and run by tests/test_oracle_sanitize.py.
 * Prints "sanitize ok" and exits 0 when every call returned normally and the results are finite.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

void orc_matmul_nn(const double*, const double*, double*, int, int, int);
void orc_matmul_tn(const double*, const double*, double*, int, int, int);
void orc_matmul_nt(const double*, const double*, double*, int, int, int);
int orc_project_core(const double*, const double*, const double*, double*, int, int, int);
void orc_core_average(const double*, double*, int, int);
void orc_adam_core(const double*, double*, double*, double*, long, int, double, double, double);
void orc_sgd_core(const double*, double*, double*, long, double);
int orc_backproject_apply(double*, const double*, const double*, const double*, int, int, int, double, double, double);
int orc_householder_qr(const double*, double*, double*, int, int);
int orc_jacobi_svd(const double*, double*, double*, double*, int, int);
int orc_refresh_rsvd(const double*, const double*, double*, double*, double*, double*, int, int, int, int, int);

static unsigned long long state = 88172645463325252ULL;
static double rnd(void) {                      /* xorshift: inputs only */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}
static double* mat(size_t count, int fill) {
    double* p = (double*)malloc(sizeof(double) * (count ? count : 1));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (size_t i = 0; i < count; ++i) p[i] = fill ? rnd() : 0.0;
    return p;
}
static int finite(const double* p, size_t count) {
    for (size_t i = 0; i < count; ++i) if (!isfinite(p[i])) return 0;
    return 1;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int one_case(int m, int n, int r, int p, int q, int workers) {
    const int k = r + p;
    double *G = mat((size_t)m * n, 1), *U = mat((size_t)m * r, 1), *V = mat((size_t)n * r, 1);
    double *C = mat((size_t)r * r, 0), *Cs = mat((size_t)workers * r * r, 1), *Cbar = mat((size_t)r * r, 0);
    double *M = mat((size_t)r * r, 0), *Vm = mat((size_t)r * r, 0), *D = mat((size_t)r * r, 0);
    double *W = mat((size_t)m * n, 1);
    double *A = mat((size_t)m * n, 0), *Bm = mat((size_t)n * m, 0);
    CHECK(orc_project_core(G, U, V, C, m, n, r) == 0);
    orc_core_average(Cs, Cbar, workers, r);
    for (int t = 1; t <= 3; ++t) orc_adam_core(C, M, Vm, D, (long)r * r, t, 0.9, 0.999, 1e-8);
    orc_sgd_core(C, M, D, (long)r * r, 0.9);
    CHECK(orc_backproject_apply(W, U, V, D, m, n, r, 1e-3, 0.01, 0.75) == 0);
    CHECK(finite(C, (size_t)r * r) && finite(D, (size_t)r * r) && finite(W, (size_t)m * n));
    /* products in the three orientations on the same buffers */
    orc_matmul_nn(G, V, A, m, r, n);            /* m x r in A */
    orc_matmul_tn(G, U, Bm, n, r, m);           /* n x r in Bm */
    orc_matmul_nt(U, V, A, m, n, r);            /* m x n in A */
    CHECK(finite(A, (size_t)m * n) && finite(Bm, (size_t)n * r));
    if (k <= m && k <= n) {
        double *Om = mat((size_t)n * k, 1), *Un = mat((size_t)m * r, 0), *Vn = mat((size_t)n * r, 0);
        double *sig = mat((size_t)k, 0), *Q = mat((size_t)m * k, 0), *R = mat((size_t)k * k, 0);
        double *Y = mat((size_t)m * k, 1);
        double *B = mat((size_t)k * n, 1), *Ut = mat((size_t)k * k, 0), *S = mat((size_t)k, 0), *Vt = mat((size_t)n * k, 0);
        CHECK(orc_householder_qr(Y, Q, R, m, k) == 0);
        CHECK(orc_householder_qr(Y, Q, NULL, m, k) == 0);
        CHECK(orc_jacobi_svd(B, Ut, S, Vt, k, n) >= 0);
        CHECK(orc_refresh_rsvd(G, Om, Un, Vn, sig, Q, m, n, r, p, q) == 0);
        CHECK(orc_refresh_rsvd(G, Om, Un, Vn, NULL, NULL, m, n, r, p, 0) == 0);
        CHECK(finite(Un, (size_t)m * r) && finite(Vn, (size_t)n * r) && finite(sig, (size_t)k) && finite(S, (size_t)k));
        /* rank-deficient and zero sketches */
        for (size_t i = 0; i < (size_t)m * k; ++i) Y[i] = 0.0;
        CHECK(orc_householder_qr(Y, Q, R, m, k) == 0);
        CHECK(finite(Q, (size_t)m * k));
        free(Om); free(Un); free(Vn); free(sig); free(Q); free(R); free(Y); free(B); free(Ut); free(S); free(Vt);
    } else {
        double *Om = mat((size_t)n * k, 1), *Un = mat((size_t)m * r, 0), *Vn = mat((size_t)n * r, 0);
        CHECK(orc_refresh_rsvd(G, Om, Un, Vn, NULL, NULL, m, n, r, p, q) == -2);     /* k > min(m, n): refused */
        free(Om); free(Un); free(Vn);
    }
    free(G); free(U); free(V); free(C); free(Cs); free(Cbar); free(M); free(Vm); free(D); free(W); free(A); free(Bm);
    return 0;
}

int main(void) {
    const int cases[][6] = {
        {1, 1, 1, 0, 0, 1}, {1, 9, 1, 0, 1, 2}, {9, 1, 1, 0, 1, 1}, {13, 7, 3, 2, 1, 3}, {7, 13, 3, 4, 2, 8},
        {33, 65, 17, 5, 1, 2}, {64, 31, 8, 8, 0, 1}, {12, 20, 4, 16, 1, 1}, {40, 40, 40, 0, 1, 1},
    };
    for (size_t c = 0; c < sizeof(cases) / sizeof(cases[0]); ++c)
        if (one_case(cases[c][0], cases[c][1], cases[c][2], cases[c][3], cases[c][4], cases[c][5])) {
            fprintf(stderr, "case %zu failed\n", c);
            return 1;
        }
    printf("sanitize ok\n");
    return 0;
}
