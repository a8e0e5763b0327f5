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

// Blocked variant for k <= CHB_MAXK: 32-wide block columns.  Per block column the diagonal
// block is factored and inverted in LDS, the panel below it is multiplied by that inverse and
// kept in LDS, and the trailing matrix gets its rank-32 update from the LDS panel in 4 x 4
// register tiles, so the fp64 matrix in global memory is read and written once per block
// column instead of once per column.  The inverse is assembled block row by block row from
// the inverted diagonal blocks.
constexpr int CHB = 32;
constexpr int CHB_P = CHB + 1;
constexpr int CHB_MAXK = 544;

__global__ __launch_bounds__(SMALL_THREADS) void chol_inv_blocked_kernel(const CholBlock* table, const CholBlock single,
                                                                         const double tol) {
    const CholBlock* blk = table ? table + blockIdx.x : &single;
    const int k = blk->k;
    const float* S = blk->S;
    double* A = blk->work;                     // lower triangle becomes L, S = L L^T
    double* X = blk->work + (size_t)k * k;     // X = L^-1 (lower)
    const int tid = threadIdx.x;
    const int ti = tid >> 5, tc = tid & 31;    // 32 x 32 thread grid
    __shared__ double Ld[CHB][CHB_P];
    __shared__ double Li[CHB][CHB_P];
    extern __shared__ double Pn[];             // [rows below the diagonal block][CHB_P]

    for (int idx = tid; idx < k * k; idx += SMALL_THREADS) { A[idx] = (double)S[idx]; X[idx] = 0.0; }
    __syncthreads();

    for (int J = 0; J < k; J += CHB) {
        const int jb = min(CHB, k - J);
        // ---- diagonal block -> LDS (identity padding), unblocked factorization
        Ld[ti][tc] = (ti < jb && tc < jb) ? ((tc <= ti) ? A[(size_t)(J + ti) * k + J + tc] : 0.0) : (ti == tc ? 1.0 : 0.0);
        __syncthreads();
        for (int j = 0; j < jb; ++j) {
            const double a = Ld[j][j];
            const double s0 = (double)S[(size_t)(J + j) * k + J + j];
            const bool ok = (a > 0.0) && (a > tol * s0);
            const double d = ok ? sqrt(a) : 0.0;
            const double invd = ok ? 1.0 / d : 0.0;
            __syncthreads();                                   // everyone has read the pivot
            if (tc == j && ti > j) Ld[ti][j] *= invd;
            if (tc == j && ti == j) Ld[j][j] = d;
            __syncthreads();
            if (tc > j && tc <= ti) Ld[ti][tc] -= Ld[ti][j] * Ld[tc][j];
            __syncthreads();
        }
        // ---- inverse of the diagonal block (dropped pivots: zero row and column)
        if (tid < CHB) {
            const int c = tid;                                // column c of the inverse, kept in Li[.][c]
#pragma unroll 1
            for (int i = 0; i < CHB; ++i) {
                double sacc = (i == c) ? 1.0 : 0.0;
#pragma unroll 4
                for (int j = 0; j < i; ++j) sacc -= Ld[i][j] * Li[j][c];
                const double d = Ld[i][i];
                Li[i][c] = (d != 0.0) ? sacc / d : 0.0;
            }
        }
        __syncthreads();
        if (ti < jb && tc < jb) {
            A[(size_t)(J + ti) * k + J + tc] = (tc <= ti) ? Ld[ti][tc] : 0.0;
            X[(size_t)(J + ti) * k + J + tc] = (tc <= ti) ? Li[ti][tc] : 0.0;
        }
        // ---- panel: rows below, P = A[rows, J..J+jb) Li^T
        const int r0 = J + jb;
        const int nr = k - r0;
        for (int idx = tid; idx < nr * CHB; idx += SMALL_THREADS) {
            const int i = idx >> 5, c = idx & 31;
            Pn[i * CHB_P + c] = (c < jb) ? A[(size_t)(r0 + i) * k + J + c] : 0.0;
        }
        __syncthreads();
        {
            constexpr int MAXPASS = (CHB_MAXK + CHB - 1) / CHB;
            double res[MAXPASS];
#pragma unroll
            for (int p = 0; p < MAXPASS; ++p) {
                const int i = p * CHB + ti;
                double acc = 0.0;
                if (i < nr) {
#pragma unroll 8
                    for (int j = 0; j < CHB; ++j) acc += Pn[i * CHB_P + j] * Li[tc][j];   // Li[tc][j] = 0 for j > tc
                }
                res[p] = acc;
            }
            __syncthreads();
#pragma unroll
            for (int p = 0; p < MAXPASS; ++p) {
                const int i = p * CHB + ti;
                if (i < nr) {
                    Pn[i * CHB_P + tc] = res[p];
                    if (tc < jb) A[(size_t)(r0 + i) * k + J + tc] = res[p];
                }
            }
        }
        __syncthreads();
        // ---- trailing update, lower triangle, 4 x 4 tiles: A[i][c] -= sum_j P[i][j] P[c][j]
        {
            const int T = (nr + 3) >> 2;
            const int ntile = T * (T + 1) / 2;
            for (int q = tid; q < ntile; q += SMALL_THREADS) {
                int tr = (int)((sqrt(8.0 * (double)q + 1.0) - 1.0) * 0.5);
                while ((tr + 1) * (tr + 2) / 2 <= q) ++tr;
                while (tr * (tr + 1) / 2 > q) --tr;
                const int tcx = q - tr * (tr + 1) / 2;
                const int i0 = tr * 4, c0 = tcx * 4;
                double acc[4][4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
#pragma unroll 4
                for (int j = 0; j < CHB; ++j) {
                    double pi[4], pc[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        pi[u] = (i0 + u < nr) ? Pn[(i0 + u) * CHB_P + j] : 0.0;
                        pc[u] = (c0 + u < nr) ? Pn[(c0 + u) * CHB_P + j] : 0.0;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[u][v] += pi[u] * pc[v];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int i = i0 + u, c = c0 + v;
                        if (i < nr && c <= i) A[(size_t)(r0 + i) * k + r0 + c] -= acc[u][v];
                    }
            }
        }
        __syncthreads();
    }

    // ---- off-diagonal blocks of X = L^-1, block row by block row:
    //      X[I][J] = -Li_I * sum_{K=J}^{I-1} L[I][K] X[K][J]
    const int nblk = (k + CHB - 1) / CHB;
    for (int I = 1; I < nblk; ++I) {
        const int ib = min(CHB, k - I * CHB);
        Li[ti][tc] = (ti < ib && tc < ib) ? X[(size_t)(I * CHB + ti) * k + I * CHB + tc] : 0.0;
        __syncthreads();
        for (int J = 0; J < I; ++J) {
            double sacc = 0.0;
            if (ti < ib) {
                const double* lrow = A + (size_t)(I * CHB + ti) * k;
                for (int c = J * CHB; c < I * CHB; ++c) sacc += lrow[c] * X[(size_t)c * k + J * CHB + tc];
            }
            Ld[ti][tc] = sacc;
            __syncthreads();
            if (ti < ib) {
                double v = 0.0;
#pragma unroll 8
                for (int a2 = 0; a2 < CHB; ++a2) v += Li[ti][a2] * Ld[a2][tc];       // Li lower: zero for a2 > ti
                X[(size_t)(I * CHB + ti) * k + J * CHB + tc] = -v;
            }
            __syncthreads();
        }
    }
    __syncthreads();

    // Rinv = X^T (upper triangular), fp32
    float* Rinv = blk->Rinv;
    for (int idx = tid; idx < k * k; idx += SMALL_THREADS) {
        const int a = idx / k, b = idx % k;
        Rinv[idx] = (a <= b) ? (float)X[(size_t)b * k + a] : 0.0f;
    }
    // Rtot = R Rprev with R = L^T
    double* Rtot = blk->Rtot;
    if (Rtot != nullptr) {
        const double* Rp = blk->Rprev;
        for (int idx = tid; idx < k * k; idx += SMALL_THREADS) {
            const int a = idx / k, b = idx % k;
            double sacc = 0.0;
            if (a <= b) {
                if (Rp == nullptr) {
                    sacc = A[(size_t)b * k + a];
                } else {
                    for (int c = a; c <= b; ++c) sacc += A[(size_t)c * k + a] * Rp[(size_t)c * k + b];
                }
            }
            Rtot[idx] = sacc;
        }
    }
}

hipError_t launch_chol_inv(const CholBlock* table_dev, const CholBlock* single, int blocks, int max_k, double tol,
                           hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    CholBlock sb{};
    if (single) sb = *single;
    if (max_k <= CHB_MAXK) {
        const int lds = (max_k > CHB ? max_k - CHB : 1) * CHB_P * 8;
        static thread_local bool configured = false;
        if (!configured) {
            hipError_t e = hipFuncSetAttribute((const void*)chol_inv_blocked_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (CHB_MAXK - CHB) * CHB_P * 8);
            if (e != hipSuccess) return e;
            configured = true;
        }
        hipLaunchKernelGGL(chol_inv_blocked_kernel, dim3(blocks), dim3(SMALL_THREADS), lds, stream, table_dev, sb, tol);
    } else {
        hipLaunchKernelGGL(chol_inv_kernel, dim3(blocks), dim3(SMALL_THREADS), 0, stream, table_dev, sb, tol);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ Jacobi SVD
__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

constexpr int JAC_MAX_SWEEPS = 40;

// Pair (i, j) of slot s in round rr of a round-robin tournament of n players (n even): every
// pair meets exactly once over rounds 0 .. n-2 and the pairs of one round are disjoint.
__device__ inline void tournament_pair(int n, int rr, int s, int& i, int& j) {
    i = (rr + s) % (n - 1);
    j = (s == 0) ? (n - 1) : (rr + n - 1 - s) % (n - 1);
}

// Block one-sided Jacobi on the rows of R (k x k, fp64): rows are grouped into blocks of B2/2;
// for every pair of blocks (outer tournament) the B2 rows are brought into LDS and swept once
// (inner tournament, one wave per row pair, B2/2 disjoint pairs per inner round), the B2 x B2
// product of the plane rotations is accumulated next to them and then applied to the same
// rows of Gacc.  All rotation work runs out of LDS; R and Gacc cross L2 once per block pair.
template <int B2>
__global__ __launch_bounds__(SMALL_THREADS) void jacobi_kernel(const JacobiBlock* table, const JacobiBlock single) {
    const JacobiBlock* blk = table ? table + blockIdx.x : &single;
    const int k = blk->k, r = blk->r;
    double* R = blk->R;
    double* G = blk->Gacc;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    constexpr int BH = B2 / 2;                   // rows per block
    constexpr int JAC_PER_LANE = (B2 == 32) ? 9 : SMALL_MAXK / 64;   // row elements held by one lane (k <= 576 / 1024)
    constexpr int QP = B2 + 1;                   // padded row of the rotation accumulator
    extern __shared__ double sm[];
    double* X = sm;                              // [B2][k]   rows of the block pair
    double* Q = sm + (size_t)B2 * k;             // [B2][QP]  accumulated rotations
    __shared__ int s_rot_sweep, s_rot_pair;
    __shared__ int s_grow[B2];                   // global row of each local row of the block pair, -1 = none
    __shared__ double s_sig[SMALL_MAXK];
    __shared__ int s_rank[SMALL_MAXK];
    const double tol = 1e-11;

    for (int idx = tid; idx < k * k; idx += nt) G[idx] = (idx / k == idx % k) ? 1.0 : 0.0;
    __syncthreads();

    const int nbk = (k + BH - 1) / BH;           // real blocks
    const int nbe = (nbk < 2) ? 2 : nbk + (nbk & 1);   // players of the outer tournament
    const int per = (k + 63) / 64;
    for (int sweep = 0; sweep < JAC_MAX_SWEEPS; ++sweep) {
        if (tid == 0) s_rot_sweep = 0;
        __syncthreads();
        for (int orr = 0; orr < nbe - 1; ++orr) {
            for (int os = 0; os < nbe / 2; ++os) {
                int bi, bj;
                tournament_pair(nbe, orr, os, bi, bj);
                if (bi >= nbk && bj >= nbk) continue;
                // local row l < BH: row bi*BH + l, else row bj*BH + (l - BH); -1 = no such row
                if (tid < B2) {
                    const int l = tid;
                    const int g = (l < BH) ? bi * BH + l : bj * BH + (l - BH);
                    const int bb = (l < BH) ? bi : bj;
                    s_grow[l] = (bb < nbk && g < k) ? g : -1;
                }
                __syncthreads();
                auto grow = [&](int l) -> int { return s_grow[l]; };
                for (int idx = tid; idx < B2 * k; idx += nt) {
                    const int l = idx / k, c = idx % k;
                    const int g = grow(l);
                    X[idx] = (g >= 0) ? R[(size_t)g * k + c] : 0.0;
                }
                for (int idx = tid; idx < B2 * QP; idx += nt) Q[idx] = (idx / QP == idx % QP) ? 1.0 : 0.0;
                if (tid == 0) s_rot_pair = 0;
                __syncthreads();
#pragma unroll 1
                for (int irr = 0; irr < B2 - 1; ++irr) {
                    if (wave < B2 / 2) {
                        int li, lj;
                        tournament_pair(B2, irr, wave, li, lj);
                        if (grow(li) >= 0 && grow(lj) >= 0) {
                            const int p = min(li, lj), q = max(li, lj);
                            double* xp = X + (size_t)p * k;
                            double* xq = X + (size_t)q * k;
                            double x[JAC_PER_LANE], y[JAC_PER_LANE];
                            double a = 0.0, b = 0.0, g = 0.0;
#pragma unroll
                            for (int e = 0; e < JAC_PER_LANE; ++e) {
                                const int c = lane + 64 * e;
                                if (e < per && c < k) {
                                    x[e] = xp[c]; y[e] = xq[c];
                                    a += x[e] * x[e]; b += y[e] * y[e]; g += x[e] * y[e];
                                } else {
                                    x[e] = 0.0; y[e] = 0.0;
                                }
                            }
                            a = wave_sum(a); b = wave_sum(b); g = wave_sum(g);
                            if (g != 0.0 && fabs(g) > tol * sqrt(a * b)) {
                                const double zeta = (b - a) / (2.0 * g);
                                const double t = ((zeta >= 0.0) ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                                const double cs = 1.0 / sqrt(1.0 + t * t);
                                const double sn = cs * t;
#pragma unroll
                                for (int e = 0; e < JAC_PER_LANE; ++e) {
                                    const int c = lane + 64 * e;
                                    if (e < per && c < k) {
                                        xp[c] = cs * x[e] - sn * y[e];
                                        xq[c] = sn * x[e] + cs * y[e];
                                    }
                                }
                                if (lane < B2) {
                                    const double u = Q[p * QP + lane], v = Q[q * QP + lane];
                                    Q[p * QP + lane] = cs * u - sn * v;
                                    Q[q * QP + lane] = sn * u + cs * v;
                                }
                                if (lane == 0) atomicAdd(&s_rot_pair, 1);
                            }
                        }
                    }
                    __syncthreads();
                }
                if (s_rot_pair != 0) {
                    // rows back to R; the same combination of rows applied to Gacc
                    for (int idx = tid; idx < B2 * k; idx += nt) {
                        const int l = idx / k, c = idx % k;
                        const int g = grow(l);
                        if (g >= 0) R[(size_t)g * k + c] = X[idx];
                    }
                    __syncthreads();                         // X is free from here on
                    constexpr int RG = 4;                    // thread groups sharing the output rows
                    constexpr int OUT = B2 / RG;
                    const int rg = tid / (SMALL_THREADS / RG);
                    for (int c = tid % (SMALL_THREADS / RG); c < k; c += SMALL_THREADS / RG) {
                        double acc[OUT];
#pragma unroll
                        for (int o = 0; o < OUT; ++o) acc[o] = 0.0;
#pragma unroll 1
                        for (int j0 = 0; j0 < B2; j0 += 8) {
                            double gv[8];
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                const int g = grow(j0 + j);
                                gv[j] = (g >= 0) ? G[(size_t)g * k + c] : 0.0;
                            }
#pragma unroll
                            for (int o = 0; o < OUT; ++o)
#pragma unroll
                                for (int j = 0; j < 8; ++j) acc[o] += Q[(rg * OUT + o) * QP + j0 + j] * gv[j];
                        }
                        // every group reads all B2 rows of Gacc, so the new rows are parked in LDS
                        // and written to Gacc only after the barrier below
#pragma unroll
                        for (int o = 0; o < OUT; ++o) {
                            const int l = rg * OUT + o;
                            if (grow(l) >= 0) X[(size_t)l * k + c] = acc[o];
                        }
                    }
                    __syncthreads();
                    for (int idx = tid; idx < B2 * k; idx += nt) {
                        const int l = idx / k, c = idx % k;
                        const int g = grow(l);
                        if (g >= 0) G[(size_t)g * k + c] = X[idx];
                    }
                    if (tid == 0) s_rot_sweep += s_rot_pair;
                }
                __syncthreads();
            }
        }
        const int rotated = s_rot_sweep;
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

// max_k: largest k of the launch (sizes the LDS row buffer)
hipError_t launch_jacobi(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, int max_k,
                         hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    JacobiBlock sb{};
    if (single) sb = *single;
    typedef void (*fn_t)(const JacobiBlock*, const JacobiBlock);
    // 32 rows per block pair while they fit in the 160 KB of LDS next to the static arrays
    // (about 13 KB), else 16
    const size_t budget = 160 * 1024 - 14 * 1024;
    const bool big = (size_t)32 * max_k * 8 + 32 * 33 * 8 <= budget;
    fn_t fn = big ? jacobi_kernel<32> : jacobi_kernel<16>;
    const int b2 = big ? 32 : 16;
    const int lds = b2 * max_k * 8 + b2 * (b2 + 1) * 8;
    if ((size_t)lds > budget) return hipErrorInvalidValue;
    static thread_local int configured[2] = {0, 0};       // largest dynamic LDS size set so far
    if (configured[big ? 1 : 0] < lds) {
        hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        configured[big ? 1 : 0] = lds;
    }
    hipLaunchKernelGGL(fn, dim3(blocks), dim3(SMALL_THREADS), lds, stream, table_dev, sb);
    return hipGetLastError();
}

}  // namespace tsr
