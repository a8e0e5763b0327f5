// Element-wise kernels on the r x r cores and the small fp64 factorizations used by the
// subspace refresh (Cholesky + triangular inverse for the thin QR, one-sided Jacobi SVD).
#include "small.h"

namespace tsr {

// ------------------------------------------------------------------ Adam on the core
// m <- b1 m + (1-b1) c ; v <- b2 v + (1-b2) c^2 ; d = (m/c1) / (sqrt(v/c2) + eps)
__global__ __launch_bounds__(256) void adam_kernel(const CoreBlock* table, const CoreBlock single,
                                                   const AdamScalars s) {
    const CoreBlock* b = table ? table + blockIdx.y : &single;
    const float* C = b->C;
    float* __restrict__ M = b->M;
    float* __restrict__ Vm = b->Vm;
    float* D = b->D;
    const long long n = b->count;
    const float omb1 = 1.0f - s.beta1, omb2 = 1.0f - s.beta2;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x) {
        const float g = C[i];
        const float m = s.beta1 * M[i] + omb1 * g;
        const float v = s.beta2 * Vm[i] + omb2 * (g * g);
        M[i] = m;
        Vm[i] = v;
        D[i] = (m * s.inv_c1) / (sqrtf(v * s.inv_c2) + s.eps);
    }
}

hipError_t launch_adam(const CoreBlock* table_dev, const CoreBlock* single, int blocks, long long max_count,
                       const AdamScalars& s, hipStream_t stream) {
    if (blocks <= 0 || max_count <= 0) return hipSuccess;
    long long bx = (max_count + 255) / 256;
    if (bx > 2048) bx = 2048;
    CoreBlock sb{};
    if (single) sb = *single;
    hipLaunchKernelGGL(adam_kernel, dim3((unsigned)bx, blocks), dim3(256), 0, stream, table_dev, sb, s);
    return hipGetLastError();
}

// 32 x 32 patch per workgroup (256 threads = 32 x 8): coalesced reads and writes of the fp32
// arrays, LDS transpose for the bf16 D^T.
__global__ __launch_bounds__(256) void adam_t_kernel(const AdamTBlock* table, const AdamScalars s) {
    const AdamTBlock b = table[blockIdx.z];
    const int r = b.r;
    const int row0 = blockIdx.y * 32, col0 = blockIdx.x * 32;
    if (row0 >= r || col0 >= r) return;
    __shared__ unsigned short tile[32][34];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const float omb1 = 1.0f - s.beta1, omb2 = 1.0f - s.beta2;
    for (int i = ty; i < 32; i += 8) {
        const int row = row0 + i, col = col0 + tx;
        float d = 0.0f;
        if (row < r && col < r) {
            const long long idx = (long long)row * r + col;
            const float g = b.C[idx];
            const float m = s.beta1 * b.M[idx] + omb1 * g;
            const float v = s.beta2 * b.Vm[idx] + omb2 * (g * g);
            b.M[idx] = m;
            b.Vm[idx] = v;
            d = (m * s.inv_c1) / (sqrtf(v * s.inv_c2) + s.eps);
            b.D[idx] = d;
        }
        __bf16 h = (__bf16)d;
        tile[i][tx] = __builtin_bit_cast(unsigned short, h);
        if (b.Db && row < r && col < r) ((unsigned short*)b.Db)[(long long)row * b.ldt + col] = tile[i][tx];
    }
    __syncthreads();
    unsigned short* DT = (unsigned short*)b.DTb;
    unsigned short* DF = (unsigned short*)b.DTf;
    const int ksteps = r / 16;
    for (int i = ty; i < 32; i += 8) {
        const int trow = col0 + i, tcol = row0 + tx;     // D^T[col][row]
        if (trow < r && tcol < r) {
            if (DF) DF[(((long long)(trow / 32) * ksteps + tcol / 16) * 64 + ((tcol % 16) / 8) * 32 + trow % 32) * 8 + tcol % 8] = tile[tx][i];
            else DT[(long long)trow * b.ldt + tcol] = tile[tx][i];
        }
    }
}

hipError_t launch_adam_t(const AdamTBlock* table_dev, int blocks, int max_r, const AdamScalars& s,
                         hipStream_t stream) {
    if (blocks <= 0 || max_r <= 0) return hipSuccess;
    const int g = (max_r + 31) / 32;
    hipLaunchKernelGGL(adam_t_kernel, dim3(g, g, blocks), dim3(256), 0, stream, table_dev, s);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void sgd_kernel(const float* C, float* M, float* D, long long n, float beta) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x) {
        const float m = beta * M[i] + (1.0f - beta) * C[i];
        M[i] = m;
        D[i] = m;
    }
}

hipError_t launch_sgd(const float* C, float* M, float* D, long long count, float beta, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    long long bx = (count + 255) / 256;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)bx), dim3(256), 0, stream, C, M, D, count, beta);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void average_kernel(const float* Cs, int K, long long n, float* out) {
    const float inv = 1.0f / (float)K;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (long long)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int w = 0; w < K; ++w) s += Cs[(long long)w * n + i];
        out[i] = s * inv;
    }
}

hipError_t launch_average(const float* Cs, int K, long long count, float* out, hipStream_t stream) {
    if (count <= 0) return hipSuccess;
    long long bx = (count + 255) / 256;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(average_kernel, dim3((unsigned)bx), dim3(256), 0, stream, Cs, K, count, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ helpers of the exact-SVD refresh
// out (k x k fp32) = identity
__global__ __launch_bounds__(256) void identity_kernel(float* out, int k) {
    const long long n = (long long)k * k;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
        out[i] = (i / k == i % k) ? 1.0f : 0.0f;
}

hipError_t launch_identity(float* out, int k, hipStream_t stream) {
    if (k <= 0) return hipSuccess;
    long long bx = ((long long)k * k + 255) / 256;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(identity_kernel, dim3((unsigned)bx), dim3(256), 0, stream, out, k);
    return hipGetLastError();
}

// The gradient as a tall contiguous fp32 matrix: out = G (rows x cols -> rows x cols) or, with
// transpose, out = G^T (cols x rows), through a 32 x 33 LDS tile so that both sides are coalesced.
template <bool BF16>
__global__ __launch_bounds__(256) void tall_copy_kernel(const void* G, long long ldg, int rows, int cols, int transpose,
                                                        float* out) {
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int i = ty; i < 32; i += 8) {
        const int r = r0 + i, c = c0 + tx;
        float v = 0.0f;
        if (r < rows && c < cols) {
            if constexpr (BF16) v = __uint_as_float(((unsigned)((const unsigned short*)G)[(long long)r * ldg + c]) << 16);
            else v = ((const float*)G)[(long long)r * ldg + c];
        }
        tile[i][tx] = v;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        if (transpose) {
            const int c = c0 + i, r = r0 + tx;             // out[c][r]
            if (c < cols && r < rows) out[(long long)c * rows + r] = tile[tx][i];
        } else {
            const int r = r0 + i, c = c0 + tx;
            if (r < rows && c < cols) out[(long long)r * cols + c] = tile[i][tx];
        }
    }
}

hipError_t launch_tall_copy(const void* G, int g_bf16, long long ldg, int rows, int cols, int transpose, float* out,
                            hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    dim3 grid((cols + 31) / 32, (rows + 31) / 32);
    if (g_bf16) hipLaunchKernelGGL(tall_copy_kernel<true>, grid, dim3(256), 0, stream, G, ldg, rows, cols, transpose, out);
    else hipLaunchKernelGGL(tall_copy_kernel<false>, grid, dim3(256), 0, stream, G, ldg, rows, cols, transpose, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ stream calibration
typedef __attribute__((ext_vector_type(4))) float f32x4_s;
__global__ __launch_bounds__(256) void stream_kernel(f32x4_s* dst, const f32x4_s* src, long long n4, float scale) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
         i += (long long)gridDim.x * blockDim.x) {
        f32x4_s v = src[i];
        dst[i] = v * scale;
    }
}

hipError_t launch_stream(float* dst, const float* src, long long count, float scale, hipStream_t stream) {
    const long long n4 = count / 4;
    if (n4 <= 0) return hipSuccess;
    long long bx = (n4 + 255) / 256;
    if (bx > 256 * 32) bx = 256 * 32;
    hipLaunchKernelGGL(stream_kernel, dim3((unsigned)bx), dim3(256), 0, stream, (f32x4_s*)dst, (const f32x4_s*)src, n4,
                       scale);
    return hipGetLastError();
}

// ------------------------------------------------------------------ Cholesky + inverse
constexpr int SMALL_THREADS = 1024;
constexpr int SMALL_MAXK = 1024;

// shift_rel * (largest diagonal entry of the k x k fp32 matrix S), computed by the whole workgroup
__device__ inline double diagonal_shift(const float* S, int k, double shift_rel) {
    __shared__ double s_wave_max[SMALL_THREADS / 64];
    __shared__ double s_shift;
    const int tid = threadIdx.x, nt = blockDim.x;
    double mx = 0.0;
    for (int j = tid; j < k; j += nt) mx = fmax(mx, (double)S[(size_t)j * k + j]);
    for (int off = 32; off > 0; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off));
    if ((tid & 63) == 0) s_wave_max[tid >> 6] = mx;
    __syncthreads();
    if (tid == 0) {
        double m = 0.0;
        for (int w = 0; w < (nt >> 6); ++w) m = fmax(m, s_wave_max[w]);
        s_shift = shift_rel * m;
    }
    __syncthreads();
    return s_shift;
}

__global__ __launch_bounds__(SMALL_THREADS) void chol_inv_kernel(const CholBlock* table, const CholBlock single,
                                                                 const double tol, const double shift_rel) {
    const CholBlock* blk = table ? table + blockIdx.x : &single;
    const int k = blk->k;
    const float* S = blk->S;
    double* A = blk->work;                     // lower triangle becomes L, S = L L^T
    double* X = blk->work + (size_t)k * k;     // X = L^-1 (lower)
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ double colj[SMALL_MAXK];
    __shared__ double s_invd;

    const double shift = diagonal_shift(S, k, shift_rel);
    for (int idx = tid; idx < k * k; idx += nt) A[idx] = (double)S[idx] + ((idx / k == idx % k) ? shift : 0.0);
    __syncthreads();

    for (int j = 0; j < k; ++j) {
        if (tid == 0) {
            const double a = A[(size_t)j * k + j];
            const double s0 = (double)S[(size_t)j * k + j];
            if (a > 0.0 && a > tol * s0) {
                const double d = sqrt(a);
                A[(size_t)j * k + j] = d;
                s_invd = 1.0 / d;
            } else {                            // dependent column: drop it
                A[(size_t)j * k + j] = 0.0;
                s_invd = 0.0;
            }
        }
        __syncthreads();
        const double invd = s_invd;
        for (int i = j + 1 + tid; i < k; i += nt) {
            const double v = A[(size_t)i * k + j] * invd;
            A[(size_t)i * k + j] = v;
            colj[i] = v;
        }
        __syncthreads();
        if (invd != 0.0) {
            for (int i = j + 1 + wave; i < k; i += nw) {
                const double li = colj[i];
                double* row = A + (size_t)i * k;
                for (int c = j + 1 + lane; c <= i; c += 64) row[c] -= li * colj[c];
            }
        }
        __syncthreads();
    }

    // X = L^-1 by forward substitution, one column per thread (entries above the diagonal
    // come out as exact zeros, which keeps every lane on the same (i, j))
    for (int c = tid; c < k; c += nt) {
        for (int i = 0; i < k; ++i) {
            double s = (i == c) ? 1.0 : 0.0;
            const double* row = A + (size_t)i * k;
            for (int j = 0; j < i; ++j) s -= row[j] * X[(size_t)j * k + c];
            const double d = row[i];
            X[(size_t)i * k + c] = (d != 0.0) ? s / d : 0.0;
        }
    }
    __syncthreads();

    // Rinv = X^T (upper triangular), fp32
    float* Rinv = blk->Rinv;
    for (int idx = tid; idx < k * k; idx += nt) {
        const int a = idx / k, b = idx % k;
        Rinv[idx] = (a <= b) ? (float)X[(size_t)b * k + a] : 0.0f;
    }
    // Rtot = R = L^T
    double* Rtot = blk->Rtot;
    if (Rtot != nullptr) {
        for (int idx = tid; idx < k * k; idx += nt) {
            const int a = idx / k, b = idx % k;
            Rtot[idx] = (a <= b) ? A[(size_t)b * k + a] : 0.0;
        }
    }
}

// Blocked variant for k <= CHB_MAXK, three launches.  First (this kernel, one workgroup per
// matrix): 32-wide block columns; per block column the diagonal block is factored and inverted
// in LDS, the panel below it is multiplied by that inverse and kept in LDS, and the trailing
// matrix gets its rank-32 update from the LDS panel (fp64 MFMAs), so the fp64 matrix in global
// memory is read and written once per block column instead of once per column.  It leaves L in
// the lower triangle of `work` and the inverted diagonal blocks in the second k x k of `work`;
// chol_inverse_kernel then forms the blocks of L^-1 below the diagonal and chol_output_kernel
// writes R^-1 (fp32) and R.
__device__ inline double readlane_f64(double v, int lane) {      // lane: a compile-time constant
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

constexpr int CHB = 32;
constexpr int CHB_P = CHB + 1;
constexpr int CHB_MAXK = 544;

__global__ __launch_bounds__(SMALL_THREADS) void chol_inv_blocked_kernel(const CholBlock* table, const CholBlock single,
                                                                         const double tol, const double shift_rel) {
    const CholBlock* blk = table ? table + blockIdx.x : &single;
    const int k = blk->k;
    const float* S = blk->S;
    double* A = blk->work;                     // lower triangle becomes L, S = L L^T
    double* X = blk->work + (size_t)k * k;     // X = L^-1 (lower)
    const int tid = threadIdx.x;
    const int ti = tid >> 5, tc = tid & 31;    // 32 x 32 thread grid
    typedef double d4_t __attribute__((ext_vector_type(4)));
    const int wv = tid >> 6, li16 = tid & 15, lk4 = (tid & 63) >> 4;      // wave; MFMA lane coordinates
    __shared__ double Ld[CHB][CHB_P];
    __shared__ double Li[CHB][CHB_P];
    __shared__ double s_invd[CHB];             // reciprocal diagonal of the current diagonal block
    extern __shared__ double Pn[];             // [block rows * CHB][CHB_P]

    // (X is written where it is read: diagonal blocks whole, the blocks below them in the inverse phase)
    const double shift = diagonal_shift(S, k, shift_rel);
    for (int idx = tid; idx < k * k; idx += SMALL_THREADS) A[idx] = (double)S[idx] + ((idx / k == idx % k) ? shift : 0.0);
    __syncthreads();

    for (int J = 0; J < k; J += CHB) {
        const int jb = min(CHB, k - J);
        // ---- diagonal block -> LDS (identity padding), unblocked factorization
        Ld[ti][tc] = (ti < jb && tc < jb) ? ((tc <= ti) ? A[(size_t)(J + ti) * k + J + tc] : 0.0) : (ti == tc ? 1.0 : 0.0);
        __syncthreads();
        // One wave factors the 32 x 32 block, right-looking: lane i owns row i in registers; at
        // step j the pivot is read from lane j, and every lane updates the rest of its row with
        // the entries of column j read from their lanes (independent multiply-adds, no serial
        // chain beyond the pivot's reciprocal square root).
        if (tid < 64) {
            const int i = tid & 31;
            const bool act = tid < CHB;
            double arow[CHB];
#pragma unroll
            for (int c = 0; c < CHB; ++c) arow[c] = Ld[i][c];
            const double sdiag = (i < jb) ? (double)S[(size_t)(J + i) * k + J + i] : 1.0;
#pragma unroll
            for (int j = 0; j < CHB; ++j) {
                const double piv = readlane_f64(arow[j], j);
                const double s0 = readlane_f64(sdiag, j);
                const bool ok = (piv > 0.0) && (piv > tol * s0);
                const double pp = ok ? piv : 1.0;
                double rinv = __builtin_amdgcn_rsq(pp);
                const double hh = 0.5 * pp;
                rinv = rinv * (1.5 - hh * rinv * rinv);
                rinv = rinv * (1.5 - hh * rinv * rinv);
                const double invd = ok ? rinv : 0.0;
                const double lij = (i > j) ? arow[j] * invd : ((i == j) ? pp * invd : 0.0);
                arow[j] = lij;
                if (act) { if (i >= j) Ld[i][j] = lij; if (i == j) s_invd[j] = invd; }
#pragma unroll
                for (int c = j + 1; c < CHB; ++c) arow[c] -= lij * readlane_f64(lij, c);
            }
        }
        __syncthreads();
        // ---- inverse of the diagonal block (dropped pivots: zero row and column), by halves:
        // the four 8 x 8 diagonal sub-blocks by forward substitution (a column per lane), then the
        // blocks below them from  X21 = -X22 (L21 X11)  at sizes 8 and 16, every entry of a product
        // on its own thread; the panel buffer (free at this point) holds the inner products.
        Li[ti][tc] = 0.0;
        __syncthreads();
        if (tid < CHB) {
            const int d0 = tid & ~7, c = tid & 7;             // sub-block origin, column inside it
            double xc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                double sa = (i == c) ? 1.0 : 0.0;
#pragma unroll
                for (int j = 0; j < i; ++j) sa -= Ld[d0 + i][d0 + j] * xc[j];
                xc[i] = sa * s_invd[d0 + i];
                Li[d0 + i][d0 + c] = xc[i];
            }
        }
        __syncthreads();
#pragma unroll
        for (int half = 8; half <= 16; half *= 2) {
            // pairs of neighbouring diagonal blocks of size `half`: rows r0 + half .., columns r0 ..
            const int npair = CHB / (2 * half);
            const int per = half * half;
            const bool mine = tid < npair * per;
            const int pr = tid / per, e = tid % per;
            const int i = e / half, c = e % half;
            const int o = pr * 2 * half;                      // origin of the pair
            if (mine) {
                double m = 0.0;                               // (L21 X11)[i][c]
                for (int j = c; j < half; ++j) m += Ld[o + half + i][o + j] * Li[o + j][o + c];
                Pn[(o + half + i) * CHB_P + o + c] = m;
            }
            __syncthreads();
            if (mine) {
                double x = 0.0;                               // (X22 M)[i][c]
                for (int j = 0; j <= i; ++j) x += Li[o + half + i][o + half + j] * Pn[(o + half + j) * CHB_P + o + c];
                Li[o + half + i][o + c] = -x;
            }
            __syncthreads();
        }
        if (ti < jb && tc < jb) {
            A[(size_t)(J + ti) * k + J + tc] = (tc <= ti) ? Ld[ti][tc] : 0.0;
            X[(size_t)(J + ti) * k + J + tc] = (tc <= ti) ? Li[ti][tc] : 0.0;
        }
        // ---- panel: rows below, P = A[rows, J..J+jb) Li^T, on fp64 MFMAs (lane l supplies
        // A[l % 16][l / 16] and B[l / 16][l % 16], receives D[4 v + l / 16][l % 16]): 16-row
        // tiles dealt to the waves, the rows of A straight from global memory, Li^T from LDS.
        // P goes back to A and stays in the panel buffer (rows past the matrix: zeros).
        const int r0 = J + jb;
        const int nr = k - r0;
        const int nrt = (nr + 15) >> 4;
        for (int t = wv; t < nrt; t += SMALL_THREADS / 64) {       // one wave reads and rewrites its 16 rows
            const int i0 = t * 16;
            const int row = i0 + li16;
            const double* arow_g = A + (size_t)(r0 + min(row, nr - 1)) * k + J;
            d4_t acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
            double a[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int c = 4 * q + lk4;
                a[q] = (row < nr && c < jb) ? arow_g[min(c, jb - 1)] : 0.0;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a[q], Li[li16][4 * q + lk4], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a[q], Li[16 + li16][4 * q + lk4], acc1, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + 4 * v + lk4;
                Pn[i * CHB_P + li16] = acc0[v];
                Pn[i * CHB_P + 16 + li16] = acc1[v];
                if (i < nr && li16 < jb) A[(size_t)(r0 + i) * k + J + li16] = acc0[v];
                if (i < nr && 16 + li16 < jb) A[(size_t)(r0 + i) * k + J + 16 + li16] = acc1[v];
            }
        }
        __syncthreads();
        // ---- trailing update, lower triangle by 16 x 16 tiles: A[i][c] -= sum_j P[i][j] P[c][j]
        {
            const int ntile = nrt * (nrt + 1) / 2;
            for (int q = wv; q < ntile; q += SMALL_THREADS / 64) {
                int tr = (int)((sqrtf(8.0f * (float)q + 1.0f) - 1.0f) * 0.5f);
                while ((tr + 1) * (tr + 2) / 2 <= q) ++tr;
                while (tr * (tr + 1) / 2 > q) --tr;
                const int tcx = q - tr * (tr + 1) / 2;
                const int i0 = tr * 16, c0 = tcx * 16;
                const double* pa = Pn + (size_t)(i0 + li16) * CHB_P + lk4;
                const double* pb = Pn + (size_t)(c0 + li16) * CHB_P + lk4;
                d4_t acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(pa[4 * u], pb[4 * u], acc, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int i = i0 + 4 * v + lk4, c = c0 + li16;
                    if (i < nr && c <= i) A[(size_t)(r0 + i) * k + r0 + c] -= acc[v];
                }
            }
        }
        __syncthreads();
    }
}

// Second launch of the blocked variant: the blocks of X = L^-1 below the diagonal, block column by
// block column (forward substitution with 32 right-hand sides):
//     X[I][J] = -Li_I * sum_{K=J}^{I-1} L[I][K] X[K][J].
// Block columns are independent; CHOL_INV_SPLIT workgroups per matrix share them (column J costs
// about nblk - 1 - J block rows, so they are dealt from both ends).  The block column of X stays
// in LDS (block K - J at rows (K - J) * 32); the 32 x 32 products run on fp64 MFMAs
// (v_mfma_f64_16x16x4: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16], receives
// D[4 v + l / 16][l % 16]), one 16 x 16 tile per wave, the blocks of L straight from global memory.
constexpr int CHOL_INV_SPLIT = 3;
__global__ __launch_bounds__(256) void chol_inverse_kernel(const CholBlock* table, const CholBlock single, const int n_blocks) {
    const int b = blockIdx.x / CHOL_INV_SPLIT, part = blockIdx.x % CHOL_INV_SPLIT;
    if (b >= n_blocks) return;
    CholBlock cb = single;
    if (table) cb = table[b];
    const int k = cb.k;
    const double* A = cb.work;                 // L in the lower triangle
    double* X = cb.work + (size_t)k * k;       // diagonal blocks hold the inverted diagonal blocks of L
    typedef double d4_t __attribute__((ext_vector_type(4)));
    const int tid = threadIdx.x;
    const int wv = tid >> 6, li16 = tid & 15, lk4 = (tid & 63) >> 4;
    const int tr = (wv >> 1) & 1, tcb = wv & 1;
    __shared__ double Ld[CHB][CHB_P];
    extern __shared__ double Pn[];             // [block rows * CHB][CHB_P]
    const int nblk = (k + CHB - 1) / CHB;
    const int ncol = nblk - 1;                 // block columns with blocks below the diagonal
    // columns 0, 1, 2, ... go to parts 0, 1, 2, 2, 1, 0, 0, 1, ...: long and short columns mix
    for (int J = 0; J < ncol; ++J) {
        const int pos = J % (2 * CHOL_INV_SPLIT);
        const int owner = (pos < CHOL_INV_SPLIT) ? pos : 2 * CHOL_INV_SPLIT - 1 - pos;
        if (owner != part) continue;           // uniform over the workgroup
        for (int e = tid; e < CHB * CHB; e += 256)
            Pn[(e >> 5) * CHB_P + (e & 31)] = X[(size_t)(J * CHB + (e >> 5)) * k + J * CHB + (e & 31)];   // J < nblk - 1: a full block
        __syncthreads();
        for (int I = J + 1; I < nblk; ++I) {
            const int ib = min(CHB, k - I * CHB);
            const int lr = 16 * tr + li16;                 // this lane's row of the A operand
            const bool rok = lr < ib;
            {
                d4_t acc = {0.0, 0.0, 0.0, 0.0};
                const double* lrow = A + (size_t)(I * CHB + min(lr, ib - 1)) * k + lk4;
                // the blocks of L of this block row travel four products ahead of their use (each
                // product is eight MFMAs, far shorter than a trip to L2 or beyond)
                double an[4][8];
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    if (J + d < I) {
#pragma unroll
                        for (int q = 0; q < 8; ++q) an[d][q] = lrow[(J + d) * CHB + 4 * q];
                    }
                for (int K0 = J; K0 < I; K0 += 4) {
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const int K = K0 + d;
                        if (K < I) {                               // uniform
                            double a[8];
#pragma unroll
                            for (int q = 0; q < 8; ++q) a[q] = rok ? an[d][q] : 0.0;
                            if (K + 4 < I) {
#pragma unroll
                                for (int q = 0; q < 8; ++q) an[d][q] = lrow[(K + 4) * CHB + 4 * q];
                            }
                            const double* xb = Pn + (size_t)((K - J) * CHB + lk4) * CHB_P + 16 * tcb + li16;
#pragma unroll
                            for (int q = 0; q < 8; ++q)
                                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[q], xb[4 * q * CHB_P], acc, 0, 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) Ld[16 * tr + 4 * v + lk4][16 * tcb + li16] = acc[v];
            }
            __syncthreads();
            {
                d4_t acc = {0.0, 0.0, 0.0, 0.0};
                const double* xd = X + (size_t)(I * CHB + min(lr, ib - 1)) * k + I * CHB;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int c = 4 * q + lk4;
                    const double a = (rok && c < ib) ? xd[min(c, ib - 1)] : 0.0;     // Li_I, lower triangular
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, Ld[c][16 * tcb + li16], acc, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int r = 16 * tr + 4 * v + lk4, cc = 16 * tcb + li16;
                    const double val = -acc[v];
                    Pn[((I - J) * CHB + r) * CHB_P + cc] = val;                      // rows past the matrix: zero
                    if (r < ib) X[(size_t)(I * CHB + r) * k + J * CHB + cc] = val;
                }
            }
            __syncthreads();
        }
    }
}

// Third launch: Rinv = X^T (upper triangular, fp32) and, if asked for, Rtot = L^T (fp64), by
// 32 x 32 tiles transposed through LDS; one workgroup per tile of the output.
__global__ __launch_bounds__(256) void chol_output_kernel(const CholBlock* table, const CholBlock single, const int n_blocks,
                                                          const int tiles) {
    const int b = blockIdx.x / (tiles * tiles), t = blockIdx.x % (tiles * tiles);
    if (b >= n_blocks) return;
    CholBlock cb = single;
    if (table) cb = table[b];
    const int k = cb.k;
    const int ta = t / tiles, tb = t % tiles;      // output tile: rows ta * 32.., columns tb * 32..
    if (ta * CHB >= k || tb * CHB >= k) return;
    const double* A = cb.work;
    const double* X = cb.work + (size_t)k * k;
    __shared__ double tx[CHB][CHB_P];
    __shared__ double tl[CHB][CHB_P];
    const int tid = threadIdx.x;
    const bool upper = ta <= tb;                    // tiles below the diagonal are zero
    if (upper) {
        for (int e = tid; e < CHB * CHB; e += 256) {
            const int i = e >> 5, c = e & 31;       // source entry (tb * 32 + i, ta * 32 + c) of the lower triangles
            const int sr = tb * CHB + i, sc = ta * CHB + c;
            const bool ok = sr < k && sc < k && sc <= sr;
            tx[i][c] = ok ? X[(size_t)sr * k + sc] : 0.0;
            tl[i][c] = (ok && cb.Rtot) ? A[(size_t)sr * k + sc] : 0.0;
        }
    }
    __syncthreads();
    for (int e = tid; e < CHB * CHB; e += 256) {
        const int i = e >> 5, c = e & 31;           // output entry (ta * 32 + i, tb * 32 + c)
        const int orow = ta * CHB + i, ocol = tb * CHB + c;
        if (orow < k && ocol < k) {
            cb.Rinv[(size_t)orow * k + ocol] = upper ? (float)tx[c][i] : 0.0f;
            if (cb.Rtot) cb.Rtot[(size_t)orow * k + ocol] = upper ? tl[c][i] : 0.0;
        }
    }
}

hipError_t launch_chol_inv(const CholBlock* table_dev, const CholBlock* single, int blocks, int max_k, double tol,
                           double shift_rel, hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    CholBlock sb{};
    if (single) sb = *single;
    if (max_k <= CHB_MAXK) {
        // panel rows below the first diagonal block; in the inverse phase one block column of X
        const int pn_rows = ((max_k + CHB - 1) / CHB) * CHB;
        const int lds = pn_rows * CHB_P * 8;
        static thread_local bool configured = false;
        if (!configured) {
            hipError_t e = hipFuncSetAttribute((const void*)chol_inv_blocked_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, ((CHB_MAXK + CHB - 1) / CHB) * CHB * CHB_P * 8);
            if (e != hipSuccess) return e;
            configured = true;
        }
        hipLaunchKernelGGL(chol_inv_blocked_kernel, dim3(blocks), dim3(SMALL_THREADS), lds, stream, table_dev, sb, tol, shift_rel);
        static thread_local bool configured2 = false;
        if (!configured2) {
            hipError_t e = hipFuncSetAttribute((const void*)chol_inverse_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, ((CHB_MAXK + CHB - 1) / CHB) * CHB * CHB_P * 8);
            if (e != hipSuccess) return e;
            configured2 = true;
        }
        hipLaunchKernelGGL(chol_inverse_kernel, dim3(blocks * CHOL_INV_SPLIT), dim3(256), lds, stream, table_dev, sb, blocks);
        const int tiles = (max_k + CHB - 1) / CHB;
        hipLaunchKernelGGL(chol_output_kernel, dim3(blocks * tiles * tiles), dim3(256), 0, stream, table_dev, sb, blocks, tiles);
    } else {
        hipLaunchKernelGGL(chol_inv_kernel, dim3(blocks), dim3(SMALL_THREADS), 0, stream, table_dev, sb, tol, shift_rel);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ Jacobi SVD
__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}


// SVD of the k x k factor R through the symmetric eigenproblem of its Gram matrix, all in
// fp64 inside one workgroup:
//   T = R R^T ;  T = E diag(lambda) E^T  (Householder tridiagonalization + implicit QL with
//   accumulation of E^T) ;  rows of E^T R are mutually orthogonal with norms sigma_i.
// Squaring costs relative accuracy of singular values below 1e-8 sigma_1, far below the fp32
// data R was built from.  Compared with sweeping Jacobi rotations over full rows this needs
// about k^2 rotations in total (each applied to one k-vector held across the threads) instead
// of ~10 sweeps of k^2/2 rotations on 2k-vectors, and everything else is matrix products.
// Outputs as before: R is overwritten by E^T R, Gacc = E^T.
constexpr int QL_MAX_ITER = 60;
constexpr int JAC_PARTS = 4;            // pieces a long sum is cut into (k <= JAC_SPLIT_MAXK)
constexpr int JAC_SPLIT_MAXK = 544;
#define JAC_SPLIT_MAXK_OR(k) JAC_SPLIT_MAXK

__global__ __launch_bounds__(SMALL_THREADS) void jacobi_kernel(const JacobiBlock* table, const JacobiBlock single) {
    const JacobiBlock* blk = table ? table + blockIdx.x : &single;
    const int k = blk->k, r = blk->r;
    double* R = blk->R;
    double* W = blk->Gacc;              // rows become the eigenvectors (E^T)
    double* T = blk->tmp;               // Gram matrix, later E^T R
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ double s_d[SMALL_MAXK];      // diagonal, later eigenvalues / singular values
    __shared__ double s_e[SMALL_MAXK];      // sub-diagonal
    __shared__ double s_v[SMALL_MAXK];      // Householder vector / rotation cosines
    __shared__ double s_w[SMALL_MAXK];      // work vector / rotation sines
    __shared__ double s_rc[SMALL_MAXK];     // second buffer of rotation cosines
    __shared__ double s_rs[SMALL_MAXK];     // second buffer of rotation sines
    __shared__ double s_part[JAC_PARTS * JAC_SPLIT_MAXK];   // partial sums of the split loops
    __shared__ double s_red[SMALL_THREADS / 64];
    __shared__ int s_job[2][4];
    __shared__ int s_rank[SMALL_MAXK];

    auto block_sum = [&](double v) -> double {      // sum over the workgroup, result to all
        v = wave_sum(v);
        __syncthreads();
        if (lane == 0) s_red[wave] = v;
        __syncthreads();
        double t = 0.0;
        for (int i = 0; i < nw; ++i) t += s_red[i];
        return t;
    };

    // ---- T = R R^T (4 x 4 register tiles), W = I.  R is upper triangular: the sum for T[i][j]
    // starts at column max(i, j).  R^T goes to W first so that the tiles read along rows.
    {
        for (int idx = tid; idx < k * k; idx += nt) W[(size_t)(idx % k) * k + idx / k] = R[idx];
        __syncthreads();
        const int tiles = (k + 3) >> 2;
        for (int q = tid; q < tiles * tiles; q += nt) {
            const int i0 = (q / tiles) * 4, j0 = (q % tiles) * 4;
            if (j0 < i0) continue;                             // the mirror image is written below
            double acc[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
#pragma unroll 2
            for (int c = j0; c < k; ++c) {                     // columns before j0 hold zeros of rows j0..
                double a[4], b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a[u] = (i0 + u < k) ? W[(size_t)c * k + i0 + u] : 0.0;
                    b[u] = (j0 + u < k) ? W[(size_t)c * k + j0 + u] : 0.0;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[u][v] += a[u] * b[v];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (i0 + u < k && j0 + v < k) {
                        T[(size_t)(i0 + u) * k + j0 + v] = acc[u][v];
                        T[(size_t)(j0 + v) * k + i0 + u] = acc[u][v];
                    }
        }
        __syncthreads();
        for (int idx = tid; idx < k * k; idx += nt) W[idx] = (idx / k == idx % k) ? 1.0 : 0.0;
    }
    __syncthreads();

    // ---- Householder tridiagonalization of T (full symmetric storage), W <- H_j W as we go.
    // The two long loops of a step (the product T22 v and the update of W) have only n1 or k
    // independent outputs; each output's sum is cut into `parts` pieces so that all threads
    // carry loads (the step is bound by memory latency, not by arithmetic).
    const int parts = (k <= JAC_SPLIT_MAXK) ? JAC_PARTS : 1;
    const int tpp = nt / parts;                          // threads per part
    const int part = tid / tpp, li = tid % tpp;
    for (int j = 0; j + 2 < k; ++j) {
        const int n1 = k - j - 1;                       // length of the column below the diagonal
        // x = T[j+1.., j]; alpha = -sign(x0) |x|; v = x - alpha e1; H = I - beta v v^T
        double psum = 0.0;
        for (int i = tid; i < n1; i += nt) { const double x = T[(size_t)(j + 1 + i) * k + j]; s_v[i] = x; psum += x * x; }
        const double xnorm2 = block_sum(psum);
        const double x0 = s_v[0];
        const double xn = sqrt(xnorm2);
        double alpha = (x0 >= 0.0) ? -xn : xn;
        const double vnorm2 = xnorm2 - 2.0 * alpha * x0 + alpha * alpha;     // |x - alpha e1|^2
        const bool skip = (xnorm2 - x0 * x0 <= 0.0) || vnorm2 <= 0.0;        // already tridiagonal here
        if (skip) alpha = x0;
        __syncthreads();
        if (tid == 0) { s_d[j] = T[(size_t)j * k + j]; s_e[j] = alpha; if (!skip) s_v[0] = x0 - alpha; }
        __syncthreads();
        if (skip) continue;
        const double beta = 2.0 / vnorm2;
        const int seg = (n1 + parts - 1) / parts;
        const int c_lo = min(n1, part * seg), c_hi = min(n1, c_lo + seg);
        // p = beta T22 v   (T22 symmetric: read columns as rows, coalesced over the output index)
        for (int i = li; i < n1; i += tpp) {
            // eight independent partial sums keep eight loads in flight (the sum is a serial chain)
            double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
            const double* col = T + (size_t)(j + 1) * k + (j + 1 + i);
            int c = c_lo;
            for (; c + 8 <= c_hi; c += 8) {
                double x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = col[(size_t)(c + u) * k];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc[u] += x[u] * s_v[c + u];
            }
            for (; c < c_hi; ++c) acc[0] += col[(size_t)c * k] * s_v[c];
            s_part[part * JAC_SPLIT_MAXK_OR(k) + i] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
        }
        __syncthreads();
        double pv = 0.0;
        for (int i = tid; i < n1; i += nt) {
            double t = 0.0;
            for (int q = 0; q < parts; ++q) t += s_part[q * JAC_SPLIT_MAXK_OR(k) + i];
            t *= beta;
            s_w[i] = t;
            pv += t * s_v[i];
        }
        const double kk2 = 0.5 * beta * block_sum(pv);
        for (int i = tid; i < n1; i += nt) s_w[i] -= kk2 * s_v[i];           // w = p - (beta/2)(p.v) v
        __syncthreads();
        // T22 -= v w^T + w v^T
        for (int idx = tid; idx < n1 * n1; idx += nt) {
            const int i = idx / n1, c = idx % n1;
            T[(size_t)(j + 1 + i) * k + j + 1 + c] -= s_v[i] * s_w[c] + s_w[i] * s_v[c];
        }
        // W[j+1.., :] -= beta v (v^T W[j+1.., :]): partial column dots first ...
        for (int c = li; c < k; c += tpp) {
            const double* wc = W + (size_t)(j + 1) * k + c;
            double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
            int i = c_lo;
            for (; i + 8 <= c_hi; i += 8) {
                double x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = wc[(size_t)(i + u) * k];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc[u] += x[u] * s_v[i + u];
            }
            for (; i < c_hi; ++i) acc[0] += wc[(size_t)i * k] * s_v[i];
            s_part[part * JAC_SPLIT_MAXK_OR(k) + c] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
        }
        __syncthreads();
        // ... then every part updates its own rows
        for (int c = li; c < k; c += tpp) {
            double* wc = W + (size_t)(j + 1) * k + c;
            double y = 0.0;
            for (int q = 0; q < parts; ++q) y += s_part[q * JAC_SPLIT_MAXK_OR(k) + c];
            y *= beta;
            int i = c_lo;
            for (; i + 8 <= c_hi; i += 8) {
                double x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = wc[(size_t)(i + u) * k];
#pragma unroll
                for (int u = 0; u < 8; ++u) wc[(size_t)(i + u) * k] = x[u] - s_v[i + u] * y;
            }
            for (; i < c_hi; ++i) wc[(size_t)i * k] -= s_v[i] * y;
        }
        __syncthreads();
    }
    if (tid == 0) {
        if (k >= 2) { s_d[k - 2] = T[(size_t)(k - 2) * k + k - 2]; s_e[k - 2] = T[(size_t)(k - 1) * k + k - 2]; }
        s_d[k - 1] = T[(size_t)(k - 1) * k + k - 1];
        s_e[k - 1] = 0.0;
    }
    __syncthreads();

    // ---- implicit QL on (d, e); every rotation (c, s) of rows (i, i+1) is applied to W.
    // The scalar recurrences of a QL sweep are one serial chain and touch only (d, e); applying
    // the sweep's rotations to W touches only W.  So wave 0 produces sweeps (its lanes look for
    // the first negligible sub-diagonal entry at or after l, its lane 0 runs the recurrences,
    // operands prefetched one step ahead, the hypotenuse from a reciprocal square root, and
    // records the rotations) while the other waves apply the previous sweep to their columns of
    // W; one barrier per sweep hands the buffers over.
    {
        int l = 0, iter = 0;                              // producer state (wave 0, uniform)
        // job[b] = {m, lo, kind}; kind 1: apply rotations lo..m-1 from buffer b, 2: finished
        auto produce = [&](int b) {
            for (;;) {
                if (l >= k) { if (lane == 0) { s_job[b][2] = 2; } return; }
                int m = k - 1;
                for (int i = l + lane; i < k - 1; i += 64) {
                    const double dd = fabs(s_d[i]) + fabs(s_d[i + 1]);
                    if (fabs(s_e[i]) <= 2.3e-16 * dd) { m = i; break; }
                }
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) m = min(m, __shfl_xor(m, o, 64));
                if (m == l || iter >= QL_MAX_ITER) { ++l; iter = 0; continue; }
                ++iter;
                if (lane == 0) {
                    double* rc = b ? s_rc : s_v;
                    double* rs = b ? s_rs : s_w;
                    int lo = m;                                   // rotations recorded for rows lo .. m-1
                    double g = (s_d[l + 1] - s_d[l]) / (2.0 * s_e[l]);
                    double rr = sqrt(g * g + 1.0);
                    g = s_d[m] - s_d[l] + s_e[l] / (g + ((g >= 0.0) ? fabs(rr) : -fabs(rr)));
                    double sn = 1.0, cs = 1.0, pp = 0.0;
                    double e_i = s_e[m - 1], d_i = s_d[m - 1], d_ip1 = s_d[m];
                    bool under = false;
                    for (int i = m - 1; i >= l; --i) {
                        // next step's operands, fetched without a branch (the values read at the
                        // last step, i == l, are not used) so that the wait for them can sit
                        // at their first use, one step later
                        const int ip = max(i - 1, 0);
                        const double e_n = s_e[ip];
                        const double d_n = s_d[ip];
                        const double f = sn * e_i;
                        const double bb = cs * e_i;
                        const double h2 = f * f + g * g;
                        if (h2 == 0.0) { s_e[i + 1] = 0.0; s_d[i + 1] -= pp; s_e[m] = 0.0; under = true; break; }
                        double rinv = __builtin_amdgcn_rsq(h2);
                        const double hh = 0.5 * h2;
                        rinv = rinv * (1.5 - hh * rinv * rinv);
                        rinv = rinv * (1.5 - hh * rinv * rinv);
                        s_e[i + 1] = h2 * rinv;
                        sn = f * rinv; cs = g * rinv;
                        g = d_ip1 - pp;
                        rr = (d_i - g) * sn + 2.0 * cs * bb;
                        pp = sn * rr;
                        s_d[i + 1] = g + pp;
                        g = cs * rr - bb;
                        rc[i] = cs; rs[i] = sn;
                        lo = i;
                        d_ip1 = d_i; d_i = d_n; e_i = e_n;
                    }
                    if (!under) { s_d[l] -= pp; s_e[l] = g; s_e[m] = 0.0; }
                    s_job[b][0] = m; s_job[b][1] = lo; s_job[b][2] = 1;
                }
                // lane 0's updates of (d, e) must be visible to the whole wave's next search
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
                __builtin_amdgcn_wave_barrier();
                return;
            }
        };
        const int n_cons = nt - 64;                      // threads that apply rotations
        if (wave == 0) produce(0);
        __syncthreads();
        for (int cur = 0;; cur ^= 1) {
            const int kind = s_job[cur][2];
            if (kind == 2) break;
            if (wave == 0) {
                produce(cur ^ 1);
            } else {
                const int m = s_job[cur][0], lo = s_job[cur][1];
                const double* rc = cur ? s_rc : s_v;
                const double* rs = cur ? s_rs : s_w;
                for (int c = tid - 64; c < k; c += n_cons) {
                    double* wc = W + c;
                    double hi = wc[(size_t)m * k];                 // current row i+1, starting with i = m-1
                    int i = m - 1;
                    for (; i - 7 >= lo; i -= 8) {                  // eight rows fetched together
                        double a[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u) a[u] = wc[(size_t)(i - u) * k];
#pragma unroll
                        for (int u = 0; u < 8; ++u) {
                            const double cs = rc[i - u], sn = rs[i - u];
                            wc[(size_t)(i - u + 1) * k] = sn * a[u] + cs * hi;
                            hi = cs * a[u] - sn * hi;
                        }
                    }
                    for (; i >= lo; --i) {
                        const double cs = rc[i], sn = rs[i];
                        const double a = wc[(size_t)i * k];
                        wc[(size_t)(i + 1) * k] = sn * a + cs * hi;
                        hi = cs * a - sn * hi;
                    }
                    wc[(size_t)lo * k] = hi;
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();

    // ---- T <- W R  (rows of E^T R), 4 x 4 register tiles
    {
        const int tiles = (k + 3) >> 2;
        for (int q = tid; q < tiles * tiles; q += nt) {
            const int i0 = (q / tiles) * 4, c0 = (q % tiles) * 4;
            double acc[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
            const int jend = min(k, c0 + 4);                   // R is upper triangular
#pragma unroll 2
            for (int j = 0; j < jend; ++j) {
                double a[4], b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    a[u] = (i0 + u < k) ? W[(size_t)(i0 + u) * k + j] : 0.0;
                    b[u] = (c0 + u < k) ? R[(size_t)j * k + c0 + u] : 0.0;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[u][v] += a[u] * b[v];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (i0 + u < k && c0 + v < k) T[(size_t)(i0 + u) * k + c0 + v] = acc[u][v];
        }
    }
    __syncthreads();

    // singular values = row norms of E^T R; order descending (ties by index)
    for (int j = wave; j < k; j += nw) {
        double a = 0.0;
        for (int c = lane; c < k; c += 64) { const double v = T[(size_t)j * k + c]; a += v * v; }
        a = wave_sum(a);
        if (lane == 0) s_d[j] = sqrt(a);
    }
    __syncthreads();
    for (int j = tid; j < k; j += nt) {
        const double sj = s_d[j];
        int rank = 0;
        for (int i = 0; i < k; ++i) {
            const double si = s_d[i];
            rank += (si > sj || (si == sj && i < j)) ? 1 : 0;
        }
        s_rank[j] = rank;
        if (blk->sigma) blk->sigma[rank] = (float)sj;
    }
    __syncthreads();
    for (int j = wave; j < k; j += nw) {
        const int rank = s_rank[j];
        if (rank >= r) continue;
        const double sj = s_d[j];
        const double inv = (sj > 0.0) ? 1.0 / sj : 0.0;
        for (int c = lane; c < k; c += 64) {
            blk->XrT[(size_t)rank * k + c] = (float)(T[(size_t)j * k + c] * inv);
            blk->GrT[(size_t)rank * k + c] = (float)W[(size_t)j * k + c];
        }
    }
}

hipError_t launch_jacobi(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, int max_k,
                         hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    if (max_k > SMALL_MAXK) return hipErrorInvalidValue;
    JacobiBlock sb{};
    if (single) sb = *single;
    hipLaunchKernelGGL(jacobi_kernel, dim3(blocks), dim3(SMALL_THREADS), 0, stream, table_dev, sb);
    return hipGetLastError();
}

}  // namespace tsr
