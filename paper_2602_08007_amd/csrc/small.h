// Element-wise core kernels and the small dense factorizations of the refresh
// (internal interface).  "Batched" launches take a device table of per-block
// descriptors; with a null table the single descriptor passed by value is used.
#pragma once
#include <hip/hip_runtime.h>

namespace tsr {

// ---- Adam / momentum on the cores, core averaging
struct CoreBlock {          // one block's core arrays, `count` floats each
    const float* C; float* M; float* Vm; float* D;
    long long count;
};
struct AdamScalars { float beta1, beta2, eps, inv_c1, inv_c2; };

hipError_t launch_adam(const CoreBlock* table_dev, const CoreBlock* single, int blocks,
                       long long max_count, const AdamScalars& s, hipStream_t stream);
// Adam on square r x r cores that also writes D^T as bf16 (leading dimension ldt), the operand
// layout the bf16 lift GEMM U D = U (D^T)^T consumes.  DTf (optional, r % 32 == 0) receives D^T
// in MFMA-fragment order for the fused lift kernel: for the group g of 32 columns of D and the
// 16-wide k step s one contiguous 1 KiB record holding, for lane = 32 h + l, the 8 values
// D[16 s + 8 h ..][32 g + l].
struct AdamTBlock {
    const float* C; float* M; float* Vm; float* D;
    void* DTb; void* DTf; int r; long long ldt;
    void* Db;       // optional: D itself as bf16, r rows of pitch ldt
};
hipError_t launch_adam_t(const AdamTBlock* table_dev, int blocks, int max_r, const AdamScalars& s,
                         hipStream_t stream);
hipError_t launch_sgd(const float* C, float* M, float* D, long long count, float beta, hipStream_t stream);
hipError_t launch_average(const float* Cs, int K, long long count, float* out, hipStream_t stream);

// ---- helpers of the exact-SVD refresh: a k x k fp32 identity; the gradient (rows x cols, fp32 or
// bf16, leading dimension ldg) as a contiguous fp32 matrix, transposed (cols x rows) or not
hipError_t launch_identity(float* out, int k, hipStream_t stream);
hipError_t launch_tall_copy(const void* G, int g_bf16, long long ldg, int rows, int cols, int transpose, float* out,
                            hipStream_t stream);

// ---- plain streaming kernel dst[i] = scale * src[i] (dst may equal src): the measured HBM
// rate of the machine and the calibration of the memory-traffic counters
hipError_t launch_stream(float* dst, const float* src, long long count, float scale, hipStream_t stream);

// ---- Cholesky-based orth helper: from the k x k Gram matrix S (fp32, symmetric) of a
// tall matrix Y compute, in fp64, S = R^T R and write
//   Rinv (fp32, k x k upper) = R^-1, so that Y Rinv has orthonormal columns,
//   Rtot (fp64, k x k upper, optional) = R.
// Only the lower triangle of S is read.  A pivot at or below tol * S[j][j] marks column j as
// dependent: row/column j of Rinv and row j of Rtot become zero.  shift_rel > 0 factors
// S + shift_rel * max_j S[j][j] * I instead (shifted Cholesky QR: the factor exists whatever the
// rounding of S, no column is dropped, and Y Rinv has a condition number reduced to about
// 1 / sqrt(shift_rel); a following unshifted pass finishes the orthonormalisation).
// work = 2 k x k doubles per matrix.
struct CholBlock {
    const float* S; float* Rinv;
    double* Rtot;
    double* work;
    int k;
};
hipError_t launch_chol_inv(const CholBlock* table_dev, const CholBlock* single, int blocks, int max_k,
                           double tol, double shift_rel, hipStream_t stream);

// ---- SVD of the k x k upper-triangular factor R (fp64): an orthogonal Gacc with
// Gacc R = diag(sigma) X^T (rows mutually orthogonal), from the symmetric eigenproblem of R R^T.
// Outputs, for the r largest sigma in descending order: XrT (r x k fp32) rows x_j^T, GrT
// (r x k fp32) rows of Gacc, and sigma (k fp32, optional, all k values descending).
// Work: Gacc k x k doubles, tmp 2 k x k + 64 doubles, scratch 3 k x k + 3 k + 8 doubles (launch_eig_svd only).
struct JacobiBlock {
    double* R; double* Gacc; double* tmp;
    float* XrT; float* GrT; float* sigma;
    int k, r;
    double* scratch;
    const double* R1;
};
// R = R2 R1 for the two triangular factors of CholeskyQR2 (R2 in Gacc, result in R; fp64 MFMA)
hipError_t launch_rtot_product(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, int max_k,
                               hipStream_t stream);
// single kernel per matrix: tridiagonalization and implicit QL sweeps (any k up to 1024)
hipError_t launch_jacobi(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, int max_k,
                         hipStream_t stream);
// the same result as a chain of launches without long serial recurrences (bisection and
// inverse iteration instead of QL, chip-wide fp64 MFMA products), k <= EIG_MAXK
constexpr int EIG_MAXK = 544;
hipError_t launch_eig_svd(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, int max_k,
                          hipStream_t stream);

}  // namespace tsr
