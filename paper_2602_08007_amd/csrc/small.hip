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
    }
    __syncthreads();
    unsigned short* DT = (unsigned short*)b.DTb;
    for (int i = ty; i < 32; i += 8) {
        const int trow = col0 + i, tcol = row0 + tx;     // D^T[col][row]
        if (trow < r && tcol < r) DT[(long long)trow * b.ldt + tcol] = tile[tx][i];
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

__global__ __launch_bounds__(SMALL_THREADS) void chol_inv_kernel(const CholBlock* table, const CholBlock single,
                                                                 const double tol) {
    const CholBlock* blk = table ? table + blockIdx.x : &single;
    const int k = blk->k;
    const float* S = blk->S;
    double* A = blk->work;                     // lower triangle becomes L, S = L L^T
    double* X = blk->work + (size_t)k * k;     // X = L^-1 (lower)
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ double colj[SMALL_MAXK];
    __shared__ double s_invd;

    for (int idx = tid; idx < k * k; idx += nt) A[idx] = (double)S[idx];
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
    // Rtot = R Rprev with R = L^T
    double* Rtot = blk->Rtot;
    if (Rtot != nullptr) {
        const double* Rp = blk->Rprev;
        for (int idx = tid; idx < k * k; idx += nt) {
            const int a = idx / k, b = idx % k;
            double s = 0.0;
            if (a <= b) {
                if (Rp == nullptr) {
                    s = A[(size_t)b * k + a];
                } else {
                    for (int c = a; c <= b; ++c) s += A[(size_t)c * k + a] * Rp[(size_t)c * k + b];
                }
            }
            Rtot[idx] = s;
        }
    }
}

hipError_t launch_chol_inv(const CholBlock* table_dev, const CholBlock* single, int blocks, double tol,
                           hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    CholBlock sb{};
    if (single) sb = *single;
    hipLaunchKernelGGL(chol_inv_kernel, dim3(blocks), dim3(SMALL_THREADS), 0, stream, table_dev, sb, tol);
    return hipGetLastError();
}

// ------------------------------------------------------------------ Jacobi SVD
__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

constexpr int JAC_PER_LANE = SMALL_MAXK / 64;   // row elements held by one lane
constexpr int JAC_MAX_SWEEPS = 40;

__global__ __launch_bounds__(SMALL_THREADS) void jacobi_kernel(const JacobiBlock* table, const JacobiBlock single) {
    const JacobiBlock* blk = table ? table + blockIdx.x : &single;
    const int k = blk->k, r = blk->r;
    double* R = blk->R;
    double* G = blk->Gacc;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ int s_rot;
    __shared__ double s_sig[SMALL_MAXK];
    __shared__ int s_rank[SMALL_MAXK];
    const double tol = 1e-13;

    for (int idx = tid; idx < k * k; idx += nt) G[idx] = (idx / k == idx % k) ? 1.0 : 0.0;
    __syncthreads();

    const int kk = k + (k & 1);      // even number of players; player kk-1 may be a dummy
    const int half = kk / 2;
    const int per = (k + 63) / 64;
    for (int sweep = 0; sweep < JAC_MAX_SWEEPS; ++sweep) {
        if (tid == 0) s_rot = 0;
        __syncthreads();
        for (int rr = 0; rr < kk - 1; ++rr) {
            for (int s = wave; s < half; s += nw) {
                const int i0 = (rr + s) % (kk - 1);
                const int j0 = (s == 0) ? (kk - 1) : (rr + kk - 1 - s) % (kk - 1);
                if (i0 >= k || j0 >= k) continue;
                const int p = min(i0, j0), q = max(i0, j0);
                double* rp = R + (size_t)p * k;
                double* rq = R + (size_t)q * k;
                double x[JAC_PER_LANE], y[JAC_PER_LANE];
                double a = 0.0, b = 0.0, g = 0.0;
#pragma unroll
                for (int e = 0; e < JAC_PER_LANE; ++e) {
                    const int c = lane + 64 * e;
                    if (e < per && c < k) {
                        x[e] = rp[c]; y[e] = rq[c];
                        a += x[e] * x[e]; b += y[e] * y[e]; g += x[e] * y[e];
                    } else {
                        x[e] = 0.0; y[e] = 0.0;
                    }
                }
                a = wave_sum(a); b = wave_sum(b); g = wave_sum(g);
                if (g == 0.0 || fabs(g) <= tol * sqrt(a * b)) continue;
                const double zeta = (b - a) / (2.0 * g);
                const double t = ((zeta >= 0.0) ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                const double cs = 1.0 / sqrt(1.0 + t * t);
                const double sn = cs * t;
                double* gp = G + (size_t)p * k;
                double* gq = G + (size_t)q * k;
#pragma unroll
                for (int e = 0; e < JAC_PER_LANE; ++e) {
                    const int c = lane + 64 * e;
                    if (e < per && c < k) {
                        rp[c] = cs * x[e] - sn * y[e];
                        rq[c] = sn * x[e] + cs * y[e];
                        const double u = gp[c], v = gq[c];
                        gp[c] = cs * u - sn * v;
                        gq[c] = sn * u + cs * v;
                    }
                }
                if (lane == 0) atomicAdd(&s_rot, 1);
            }
            __syncthreads();
        }
        const int rotated = s_rot;
        __syncthreads();
        if (rotated == 0) break;
    }

    // singular values = row norms; order descending (ties by index)
    for (int j = wave; j < k; j += nw) {
        double a = 0.0;
        for (int c = lane; c < k; c += 64) { const double v = R[(size_t)j * k + c]; a += v * v; }
        a = wave_sum(a);
        if (lane == 0) s_sig[j] = sqrt(a);
    }
    __syncthreads();
    for (int j = tid; j < k; j += nt) {
        const double sj = s_sig[j];
        int rank = 0;
        for (int i = 0; i < k; ++i) {
            const double si = s_sig[i];
            rank += (si > sj || (si == sj && i < j)) ? 1 : 0;
        }
        s_rank[j] = rank;
        if (blk->sigma) blk->sigma[rank] = (float)sj;
    }
    __syncthreads();
    for (int j = wave; j < k; j += nw) {
        const int rank = s_rank[j];
        if (rank >= r) continue;
        const double sj = s_sig[j];
        const double inv = (sj > 0.0) ? 1.0 / sj : 0.0;
        for (int c = lane; c < k; c += 64) {
            blk->XrT[(size_t)rank * k + c] = (float)(R[(size_t)j * k + c] * inv);
            blk->GrT[(size_t)rank * k + c] = (float)G[(size_t)j * k + c];
        }
    }
}

hipError_t launch_jacobi(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    JacobiBlock sb{};
    if (single) sb = *single;
    hipLaunchKernelGGL(jacobi_kernel, dim3(blocks), dim3(SMALL_THREADS), 0, stream, table_dev, sb);
    return hipGetLastError();
}

}  // namespace tsr
