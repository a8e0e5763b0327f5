/*
 * CPU oracle for the TSR-Adam per-matrix optimizer path.  TEST INFRASTRUCTURE ONLY:
 * a plain, slow, fp64 restatement of the paper's update, used by the tests, the smoke
 * check and the benchmark's CPU-baseline leg to judge the GPU library.  It shares no
 * code with the GPU library and nothing in the product path may call it.
 *
 * All matrices are dense, row-major, fp64, with leading dimension = number of columns.
 * Loops are written in the order of the definitions; the only concession to speed is an
 * OpenMP "parallel for" over independent output rows of the matrix products (it does
 * not change the order in which any single output element is summed).
 *
 * What is pinned by tests that do not depend on this file (closed forms, invariants,
 * brute force, library cross-checks on tiny inputs): the matrix products, project,
 * average, Adam-on-core, lift+apply, thin QR, Jacobi SVD, the rSVD refresh.
 * Parity unpinned by any number printed in the paper: the paper gives no worked
 * numeric example of C, D, U, V or W, so every pin is a mathematical one.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- products */

/* C (M x N) = A (M x K) * B (K x N) */
void orc_matmul_nn(const double* A, const double* B, double* C, int M, int N, int K) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        double* c = C + (size_t)i * N;
        for (int j = 0; j < N; ++j) c[j] = 0.0;
        for (int k = 0; k < K; ++k) {
            const double a = A[(size_t)i * K + k];
            const double* b = B + (size_t)k * N;
            for (int j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

/* C (M x N) = A^T * B with A stored K x M, B stored K x N */
void orc_matmul_tn(const double* A, const double* B, double* C, int M, int N, int K) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        double* c = C + (size_t)i * N;
        for (int j = 0; j < N; ++j) c[j] = 0.0;
        for (int k = 0; k < K; ++k) {
            const double a = A[(size_t)k * M + i];
            const double* b = B + (size_t)k * N;
            for (int j = 0; j < N; ++j) c[j] += a * b[j];
        }
    }
}

/* C (M x N) = A * B^T with A stored M x K, B stored N x K */
void orc_matmul_nt(const double* A, const double* B, double* C, int M, int N, int K) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        const double* a = A + (size_t)i * K;
        for (int j = 0; j < N; ++j) {
            const double* b = B + (size_t)j * K;
            double s = 0.0;
            for (int k = 0; k < K; ++k) s += a[k] * b[k];
            C[(size_t)i * N + j] = s;
        }
    }
}

/* ------------------------------------------------- per-step path (Algorithm 1) */

/* Two-sided core C = U^T G V  (Section 3.3; the projection line of Algorithm 1).
 * G m x n, U m x r, V n x r, C r x r.  Returns 0, or -1 if out of memory. */
int orc_project_core(const double* G, const double* U, const double* V, double* C,
                     int m, int n, int r) {
    double* P = (double*)malloc(sizeof(double) * (size_t)m * r);
    if (!P) return -1;
    orc_matmul_nn(G, V, P, m, r, n);  /* P = G V   */
    orc_matmul_tn(U, P, C, r, r, m);  /* C = U^T P */
    free(P);
    return 0;
}

/* All-reduce average stand-in: Cbar = (1/K) sum_i C_i, summed in worker order
 * (the AR(.) operator of Algorithm 1).  Cs holds K consecutive r x r cores. */
void orc_core_average(const double* Cs, double* Cbar, int K, int r) {
    const size_t e = (size_t)r * r;
    for (size_t j = 0; j < e; ++j) {
        double s = 0.0;
        for (int i = 0; i < K; ++i) s += Cs[(size_t)i * e + j];
        Cbar[j] = s / (double)K;
    }
}

/* Adam moments and normalized update on the core (Section 3.4; the four moment /
 * bias-correction / D lines of Algorithm 1).  M, Vm updated in place, t >= 1.
 *   m <- b1 m + (1-b1) C ; v <- b2 v + (1-b2) C.C
 *   D = (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)       eps is added after the root. */
void orc_adam_core(const double* C, double* M, double* Vm, double* D, long count, int t,
                   double beta1, double beta2, double eps) {
    const double c1 = 1.0 - pow(beta1, (double)t);
    const double c2 = 1.0 - pow(beta2, (double)t);
    for (long j = 0; j < count; ++j) {
        const double g = C[j];
        M[j] = beta1 * M[j] + (1.0 - beta1) * g;
        Vm[j] = beta2 * Vm[j] + (1.0 - beta2) * (g * g);
        const double mh = M[j] / c1;
        const double vh = Vm[j] / c2;
        D[j] = mh / (sqrt(vh) + eps);
    }
}

/* Momentum-SGD variant of the core update (Algorithm 2): m <- beta m + (1-beta) C, D = m. */
void orc_sgd_core(const double* C, double* M, double* D, long count, double beta) {
    for (long j = 0; j < count; ++j) {
        M[j] = beta * M[j] + (1.0 - beta) * C[j];
        D[j] = M[j];
    }
}

/* Lift and apply (Section 3.4; last two update lines of Algorithm 1):
 *   dW = U D V^T ;  W <- W - lr (scale dW + wd W)    with the pre-update W in the decay.
 * `scale` is the scalar the experiments multiply the lifted update by (1 = Algorithm 1). */
int orc_backproject_apply(double* W, const double* U, const double* V, const double* D,
                          int m, int n, int r, double lr, double wd, double scale) {
    double* T = (double*)malloc(sizeof(double) * (size_t)m * r);
    double* dW = (double*)malloc(sizeof(double) * (size_t)m * n);
    if (!T || !dW) { free(T); free(dW); return -1; }
    orc_matmul_nn(U, D, T, m, r, r);   /* T = U D     */
    orc_matmul_nt(T, V, dW, m, n, r);  /* dW = T V^T  */
    for (size_t j = 0; j < (size_t)m * n; ++j) W[j] = W[j] - lr * (scale * dW[j] + wd * W[j]);
    free(T); free(dW);
    return 0;
}

/* ------------------------------------------------------------ thin QR (orth) */

/* Householder thin QR of Y (rows x k, rows >= k): Q (rows x k) has orthonormal columns
 * whose span contains range(Y), even when Y is rank deficient; R (k x k, may be NULL)
 * is the triangular factor with Y = Q R.  This is the orth(.) of Algorithm 1. */
int orc_householder_qr(const double* Y, double* Q, double* R, int rows, int k) {
    double* A = (double*)malloc(sizeof(double) * (size_t)rows * k);
    double* Vs = (double*)calloc((size_t)rows * k, sizeof(double)); /* reflectors, column j in Vs[:,j] */
    if (!A || !Vs) { free(A); free(Vs); return -1; }
    memcpy(A, Y, sizeof(double) * (size_t)rows * k);
    for (int j = 0; j < k; ++j) {
        double nrm2 = 0.0;
        for (int i = j; i < rows; ++i) nrm2 += A[(size_t)i * k + j] * A[(size_t)i * k + j];
        const double nrm = sqrt(nrm2);
        if (nrm == 0.0) continue;                    /* H_j = I */
        const double x0 = A[(size_t)j * k + j];
        const double alpha = (x0 >= 0.0) ? -nrm : nrm;
        /* v = x - alpha e1, normalised */
        double vn2 = 0.0;
        for (int i = j; i < rows; ++i) {
            double v = A[(size_t)i * k + j];
            if (i == j) v -= alpha;
            Vs[(size_t)i * k + j] = v;
            vn2 += v * v;
        }
        const double vn = sqrt(vn2);
        if (vn == 0.0) continue;
        for (int i = j; i < rows; ++i) Vs[(size_t)i * k + j] /= vn;
        /* A[j:, j:] <- (I - 2 v v^T) A[j:, j:] */
        for (int c = j; c < k; ++c) {
            double s = 0.0;
            for (int i = j; i < rows; ++i) s += Vs[(size_t)i * k + j] * A[(size_t)i * k + c];
            s *= 2.0;
            for (int i = j; i < rows; ++i) A[(size_t)i * k + c] -= s * Vs[(size_t)i * k + j];
        }
    }
    if (R) {
        for (int i = 0; i < k; ++i)
            for (int c = 0; c < k; ++c) R[(size_t)i * k + c] = (c >= i) ? A[(size_t)i * k + c] : 0.0;
    }
    /* Q = H_0 H_1 ... H_{k-1} [I_k; 0] : apply reflectors in reverse to the thin identity */
    for (int i = 0; i < rows; ++i)
        for (int c = 0; c < k; ++c) Q[(size_t)i * k + c] = (i == c) ? 1.0 : 0.0;
    for (int j = k - 1; j >= 0; --j) {
        for (int c = 0; c < k; ++c) {
            double s = 0.0;
            for (int i = j; i < rows; ++i) s += Vs[(size_t)i * k + j] * Q[(size_t)i * k + c];
            s *= 2.0;
            if (s != 0.0)
                for (int i = j; i < rows; ++i) Q[(size_t)i * k + c] -= s * Vs[(size_t)i * k + j];
        }
    }
    free(A); free(Vs);
    return 0;
}

/* ------------------------------------------------------------ small SVD */

/* One-sided (Hestenes) Jacobi SVD of B (k x n, k <= n), working on its rows:
 * plane rotations make the rows mutually orthogonal; then B = Ut S Vt^T with
 *   S  (k)     singular values, sorted descending,
 *   Ut (k x k) left singular vectors in columns,
 *   Vt (n x k) right singular vectors in columns (a zero column where S = 0).
 * Returns the number of sweeps used, or -1 on allocation failure. */
int orc_jacobi_svd(const double* B, double* Ut, double* S, double* Vt, int k, int n) {
    double* A = (double*)malloc(sizeof(double) * (size_t)k * n);  /* rotated rows      */
    double* J = (double*)malloc(sizeof(double) * (size_t)k * k);  /* A = J * B          */
    int* order = (int*)malloc(sizeof(int) * (size_t)k);
    double* nrm = (double*)malloc(sizeof(double) * (size_t)k);
    if (!A || !J || !order || !nrm) { free(A); free(J); free(order); free(nrm); return -1; }
    memcpy(A, B, sizeof(double) * (size_t)k * n);
    for (int i = 0; i < k; ++i)
        for (int j = 0; j < k; ++j) J[(size_t)i * k + j] = (i == j) ? 1.0 : 0.0;
    const double tol = 1e-15;
    int sweeps = 0;
    for (; sweeps < 100; ++sweeps) {
        int rotated = 0;
        for (int p = 0; p < k - 1; ++p) {
            double* ap = A + (size_t)p * n;
            for (int q = p + 1; q < k; ++q) {
                double* aq = A + (size_t)q * n;
                double alpha = 0.0, beta = 0.0, gamma = 0.0;
                for (int j = 0; j < n; ++j) {
                    alpha += ap[j] * ap[j];
                    beta += aq[j] * aq[j];
                    gamma += ap[j] * aq[j];
                }
                if (gamma == 0.0 || fabs(gamma) <= tol * sqrt(alpha * beta)) continue;
                rotated = 1;
                const double zeta = (beta - alpha) / (2.0 * gamma);
                const double tt = ((zeta >= 0.0) ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                const double c = 1.0 / sqrt(1.0 + tt * tt);
                const double s = c * tt;
                for (int j = 0; j < n; ++j) {
                    const double x = ap[j], y = aq[j];
                    ap[j] = c * x - s * y;
                    aq[j] = s * x + c * y;
                }
                double* jp = J + (size_t)p * k;
                double* jq = J + (size_t)q * k;
                for (int j = 0; j < k; ++j) {
                    const double x = jp[j], y = jq[j];
                    jp[j] = c * x - s * y;
                    jq[j] = s * x + c * y;
                }
            }
        }
        if (!rotated) break;
    }
    for (int i = 0; i < k; ++i) {
        double s = 0.0;
        for (int j = 0; j < n; ++j) s += A[(size_t)i * n + j] * A[(size_t)i * n + j];
        nrm[i] = sqrt(s);
        order[i] = i;
    }
    /* stable insertion sort, descending */
    for (int i = 1; i < k; ++i) {
        const int o = order[i];
        int j = i - 1;
        while (j >= 0 && nrm[order[j]] < nrm[o]) { order[j + 1] = order[j]; --j; }
        order[j + 1] = o;
    }
    for (int c = 0; c < k; ++c) {
        const int src = order[c];
        S[c] = nrm[src];
        /* B = J^T A, A = diag(nrm) X^T  =>  left vector c = row src of J, as a column */
        for (int i = 0; i < k; ++i) Ut[(size_t)i * k + c] = J[(size_t)src * k + i];
        for (int j = 0; j < n; ++j)
            Vt[(size_t)j * k + c] = (nrm[src] > 0.0) ? A[(size_t)src * n + j] / nrm[src] : 0.0;
    }
    free(A); free(J); free(order); free(nrm);
    return sweeps;
}

/* -------------------------------------------------- randomized-SVD refresh */

/* Subspace refresh for one worker (Section 3.5; the refresh branch of Algorithm 1, N = 1):
 *   Y = G Omega ; Q = orth(Y)
 *   q times:  Yrow = G^T Q ; Qrow = orth(Yrow) ; Y = G Qrow ; Q = orth(Y)
 *   B = Q^T G ; B = Ut S Vt^T ; U = Q Ut[:, :r] ; V = Vt[:, :r]
 * G m x n, Omega n x k (k = r + p <= min(m, n)), U m x r, V n x r,
 * sigma (k, may be NULL) singular values of B, Qout (m x k, may be NULL) final Q. */
int orc_refresh_rsvd(const double* G, const double* Omega, double* U, double* V, double* sigma,
                     double* Qout, int m, int n, int r, int p, int q) {
    const int k = r + p;
    if (k > m || k > n || r <= 0 || p < 0 || q < 0) return -2;
    double* Y = (double*)malloc(sizeof(double) * (size_t)m * k);
    double* Q = (double*)malloc(sizeof(double) * (size_t)m * k);
    double* Yrow = (double*)malloc(sizeof(double) * (size_t)n * k);
    double* Qrow = (double*)malloc(sizeof(double) * (size_t)n * k);
    double* B = (double*)malloc(sizeof(double) * (size_t)k * n);
    double* Ut = (double*)malloc(sizeof(double) * (size_t)k * k);
    double* Vt = (double*)malloc(sizeof(double) * (size_t)n * k);
    double* S = (double*)malloc(sizeof(double) * (size_t)k);
    double* Utr = (double*)malloc(sizeof(double) * (size_t)k * r);
    int rc = -1;
    if (!Y || !Q || !Yrow || !Qrow || !B || !Ut || !Vt || !S || !Utr) goto done;
    orc_matmul_nn(G, Omega, Y, m, k, n);
    if (orc_householder_qr(Y, Q, NULL, m, k)) goto done;
    for (int it = 0; it < q; ++it) {
        orc_matmul_tn(G, Q, Yrow, n, k, m);
        if (orc_householder_qr(Yrow, Qrow, NULL, n, k)) goto done;
        orc_matmul_nn(G, Qrow, Y, m, k, n);
        if (orc_householder_qr(Y, Q, NULL, m, k)) goto done;
    }
    orc_matmul_tn(Q, G, B, k, n, m);
    if (orc_jacobi_svd(B, Ut, S, Vt, k, n) < 0) goto done;
    for (int i = 0; i < k; ++i)
        for (int c = 0; c < r; ++c) Utr[(size_t)i * r + c] = Ut[(size_t)i * k + c];
    orc_matmul_nn(Q, Utr, U, m, r, k);
    for (int j = 0; j < n; ++j)
        for (int c = 0; c < r; ++c) V[(size_t)j * r + c] = Vt[(size_t)j * k + c];
    if (sigma) memcpy(sigma, S, sizeof(double) * (size_t)k);
    if (Qout) memcpy(Qout, Q, sizeof(double) * (size_t)m * k);
    rc = 0;
done:
    free(Y); free(Q); free(Yrow); free(Qrow); free(B); free(Ut); free(Vt); free(S); free(Utr);
    return rc;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of OpenMP threads the products use from now on (timing runs at one thread and at all
 * threads; no effect on any result: each output element is summed by one thread in a fixed order). */
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
