// Grouped tall-skinny GEMM on gfx950 matrix cores: 128x128 output tile per 256-thread
// workgroup, 32-deep k-tiles staged through LDS as bf16 pieces, fp32 accumulation with
// v_mfma_f32_32x32x16_bf16 (each of the 4 waves owns a 64x64 quadrant = 2x2 MFMA tiles).
//
// Global -> registers (prefetch of the next k-tile overlaps the MFMAs of the current one)
// -> split into bf16 pieces -> LDS in [row][k] order with a padded row -> 16-byte fragment
// reads.  Both operand orientations end up in the same LDS layout, so the MFMA loop is
// shared by all variants.
#include "gemm.h"

namespace tsr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int BK = 32;          // k-tile depth
constexpr int KP = BK + 8;      // padded LDS row, bf16 elements (80 bytes: 16-byte aligned rows)
constexpr int NTHREADS = 256;
constexpr int TILE_ELEMS = 128 * KP;

// ------------------------------------------------------------------ staging registers
// k-contiguous operand: each thread owns 2 chunks of 8 consecutive k of one row.
// k-strided operand:    each thread owns a 4(k) x 4(row) micro-tile.
template <bool BF16> struct StageKC;
template <> struct StageKC<false> { float v[2][8]; };
template <> struct StageKC<true> { u32x4 v[2]; };
template <bool BF16> struct StageKS;
template <> struct StageKS<false> { float v[4][4]; };
template <> struct StageKS<true> { unsigned short v[4][4]; };

__device__ inline float bf16_bits_to_float(unsigned short b) {
    return __uint_as_float(((unsigned int)b) << 16);
}

// rows x K operand, element (row, k) at p[row*ld + k]; tile rows row0..row0+127, k0..k0+31
template <bool BF16>
__device__ inline void load_kc(StageKC<BF16>& s, const void* base, long long ld, int rows,
                               int row0, int k0, int kend, bool vec_ok, int tid) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int c = tid + NTHREADS * it;
        const int grow = row0 + (c >> 2);
        const int gk = k0 + (c & 3) * 8;
        if constexpr (BF16) {
            const unsigned short* p = (const unsigned short*)base + (long long)grow * ld + gk;
            u32x4 r = {0u, 0u, 0u, 0u};
            if (grow < rows) {
                if (vec_ok && gk + 8 <= kend) {
                    r = *(const u32x4*)p;
                } else {
                    unsigned short e[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) e[j] = (gk + j < kend) ? p[j] : (unsigned short)0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) r[j] = (unsigned int)e[2 * j] | ((unsigned int)e[2 * j + 1] << 16);
                }
            }
            s.v[it] = r;
        } else {
            const float* p = (const float*)base + (long long)grow * ld + gk;
            if (grow < rows && vec_ok && gk + 8 <= kend) {
                const f32x4 a = *(const f32x4*)p;
                const f32x4 b = *(const f32x4*)(p + 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) { s.v[it][j] = a[j]; s.v[it][4 + j] = b[j]; }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) s.v[it][j] = (grow < rows && gk + j < kend) ? p[j] : 0.0f;
            }
        }
    }
}

// K x rows operand, element (row, k) at p[k*ld + row]
template <bool BF16>
__device__ inline void load_ks(StageKS<BF16>& s, const void* base, long long ld, int rows,
                               int row0, int k0, int kend, bool vec_ok, int tid) {
    const int gi = row0 + (tid & 31) * 4;
    const int kb = k0 + (tid >> 5) * 4;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int gk = kb + kk;
        if constexpr (BF16) {
            const unsigned short* p = (const unsigned short*)base + (long long)gk * ld + gi;
            if (gk < kend && vec_ok && gi + 4 <= rows) {
                const u32x2 r = *(const u32x2*)p;
                s.v[kk][0] = (unsigned short)(r[0] & 0xffffu); s.v[kk][1] = (unsigned short)(r[0] >> 16);
                s.v[kk][2] = (unsigned short)(r[1] & 0xffffu); s.v[kk][3] = (unsigned short)(r[1] >> 16);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) s.v[kk][j] = (gk < kend && gi + j < rows) ? p[j] : (unsigned short)0;
            }
        } else {
            const float* p = (const float*)base + (long long)gk * ld + gi;
            if (gk < kend && vec_ok && gi + 4 <= rows) {
                const f32x4 r = *(const f32x4*)p;
#pragma unroll
                for (int j = 0; j < 4; ++j) s.v[kk][j] = r[j];
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) s.v[kk][j] = (gk < kend && gi + j < rows) ? p[j] : 0.0f;
            }
        }
    }
}

// Write the staged k-contiguous chunks into LDS as NS bf16 pieces.
template <bool BF16, int NS>
__device__ inline void store_kc(const StageKC<BF16>& s, unsigned short* lds, int tid) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int c = tid + NTHREADS * it;
        const int off = (c >> 2) * KP + (c & 3) * 8;
        if constexpr (BF16) {
            *(u32x4*)(lds + off) = s.v[it];
        } else {
            float r[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) r[j] = s.v[it][j];
#pragma unroll
            for (int p = 0; p < NS; ++p) {
                bf16x8 h;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    h[j] = (__bf16)r[j];
                    if (p + 1 < NS) r[j] -= (float)h[j];
                }
                *(bf16x8*)(lds + p * TILE_ELEMS + off) = h;
            }
        }
    }
}

template <bool BF16, int NS>
__device__ inline void store_ks(const StageKS<BF16>& s, unsigned short* lds, int tid) {
    const int rb = (tid & 31) * 4;
    const int kb = (tid >> 5) * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int off = (rb + j) * KP + kb;
        if constexpr (BF16) {
            u32x2 w;
            w[0] = (unsigned int)s.v[0][j] | ((unsigned int)s.v[1][j] << 16);
            w[1] = (unsigned int)s.v[2][j] | ((unsigned int)s.v[3][j] << 16);
            *(u32x2*)(lds + off) = w;
        } else {
            float r[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) r[kk] = s.v[kk][j];
#pragma unroll
            for (int p = 0; p < NS; ++p) {
                bf16x4 h;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    h[kk] = (__bf16)r[kk];
                    if (p + 1 < NS) r[kk] -= (float)h[kk];
                }
                *(bf16x4*)(lds + p * TILE_ELEMS + off) = h;
            }
        }
    }
}

template <bool KS, bool BF16> struct StageSel { typedef StageKC<BF16> type; };
template <bool BF16> struct StageSel<true, BF16> { typedef StageKS<BF16> type; };

// ------------------------------------------------------------------ the kernel
template <bool A_KS, bool B_KS, bool A_BF16, int NSA, int NSB>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(const GemmLaunch L) {
    __shared__ __attribute__((aligned(16))) unsigned short sA[NSA * TILE_ELEMS];
    __shared__ __attribute__((aligned(16))) unsigned short sB[NSB * TILE_ELEMS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    int tm, tn, ks;
    const GemmProblem* pp;
    if (L.tiles != nullptr) {
        const GemmTile t = L.tiles[blockIdx.x];
        tm = t.tm; tn = t.tn; ks = t.ks;
        pp = L.probs + t.prob;
    } else {
        const int b = blockIdx.x;
        tn = b % L.tiles_n;
        tm = (b / L.tiles_n) % L.tiles_m;
        ks = b / (L.tiles_n * L.tiles_m);
        pp = &L.single;
    }
    const void* A = pp->A;
    const float* B = pp->B;
    const long long lda = pp->lda, ldb = pp->ldb, ldc = pp->ldc;
    const int M = pp->M, N = pp->N, K = pp->K;
    const float alpha = L.alpha, beta = L.beta;
    float* C = pp->C + (long long)ks * pp->c_split_stride;
    const int kbeg = ks * pp->kchunk;
    const int kend = min(K, kbeg + pp->kchunk);
    const int row0 = tm * GEMM_BM, col0 = tn * GEMM_BN;

    // vector loads need 16-byte aligned rows (8 bytes for the bf16 k-strided micro-tile)
    const int a_elem = A_BF16 ? 2 : 4;
    const bool a_vec = (((unsigned long long)A) % 16 == 0) && ((lda * a_elem) % 16 == 0);
    const bool b_vec = (((unsigned long long)B) % 16 == 0) && ((ldb * 4) % 16 == 0);

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    typename StageSel<A_KS, A_BF16>::type stA;
    typename StageSel<B_KS, false>::type stB;

    auto load_tiles = [&](int k0) {
        if constexpr (A_KS) load_ks<A_BF16>(stA, A, lda, M, row0, k0, kend, a_vec, tid);
        else load_kc<A_BF16>(stA, A, lda, M, row0, k0, kend, a_vec, tid);
        if constexpr (B_KS) load_ks<false>(stB, B, ldb, N, col0, k0, kend, b_vec, tid);
        else load_kc<false>(stB, B, ldb, N, col0, k0, kend, b_vec, tid);
    };

    if (kbeg < kend) load_tiles(kbeg);

    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        if constexpr (A_KS) store_ks<A_BF16, NSA>(stA, sA, tid);
        else store_kc<A_BF16, NSA>(stA, sA, tid);
        if constexpr (B_KS) store_ks<false, NSB>(stB, sB, tid);
        else store_kc<false, NSB>(stB, sB, tid);
        __syncthreads();
        if (k0 + BK < kend) load_tiles(k0 + BK);

#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int kofs = kk * 16 + (lane >> 5) * 8;
            bf16x8 fa[NSA][2], fb[NSB][2];
#pragma unroll
            for (int p = 0; p < NSA; ++p)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    fa[p][i] = *(const bf16x8*)(sA + p * TILE_ELEMS + (wm * 64 + i * 32 + (lane & 31)) * KP + kofs);
#pragma unroll
            for (int p = 0; p < NSB; ++p)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    fb[p][j] = *(const bf16x8*)(sB + p * TILE_ELEMS + (wn * 64 + j * 32 + (lane & 31)) * KP + kofs);
            // cross products of the pieces, smallest terms first; keep those of total order
            // below max(NSA, NSB)
            constexpr int ORD = (NSA > NSB) ? NSA : NSB;
#pragma unroll
            for (int o = ORD - 1; o >= 0; --o)
#pragma unroll
                for (int pa = 0; pa < NSA; ++pa) {
                    const int pb = o - pa;
                    if (pb < 0 || pb >= NSB) continue;
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[pa][i], fb[pb][j], acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // epilogue: lane holds column (lane & 31), rows 8*(e/4) + 4*(lane>>5) + e%4 of each 32x32 tile
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = col0 + wn * 64 + j * 32 + (lane & 31);
            const int rbase = row0 + wm * 64 + i * 32 + (lane >> 5) * 4;
            if (col >= N) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = rbase + (e >> 2) * 8 + (e & 3);
                if (row < M) {
                    float* c = C + (long long)row * ldc + col;
                    float v = alpha * acc[i][j][e];
                    if (beta != 0.0f) v += beta * (*c);
                    *c = v;
                }
            }
        }
}

// ------------------------------------------------------------------ dispatch
typedef void (*gemm_fn)(const GemmLaunch);
struct Entry { GemmVariant v; gemm_fn fn; };

#define TSR_GEMM(aks, bks, abf, nsa, nsb) \
    { {aks, bks, abf, nsa, nsb}, gemm_kernel<(aks) != 0, (bks) != 0, (abf) != 0, nsa, nsb> }

static const Entry kTable[] = {
    // A = G (k contiguous), B k-strided: G V, G Omega, G Qrow; also U D, Y Rinv, Q X
    TSR_GEMM(0, 1, 1, 1, 1), TSR_GEMM(0, 1, 1, 1, 2), TSR_GEMM(0, 1, 1, 1, 3),
    TSR_GEMM(0, 1, 0, 1, 1), TSR_GEMM(0, 1, 0, 2, 2), TSR_GEMM(0, 1, 0, 3, 3),
    // A k-strided, B k-strided: U^T P, Y^T Y, G^T Q
    TSR_GEMM(1, 1, 0, 1, 1), TSR_GEMM(1, 1, 0, 2, 2), TSR_GEMM(1, 1, 0, 3, 3),
    TSR_GEMM(1, 1, 1, 1, 1), TSR_GEMM(1, 1, 1, 1, 2), TSR_GEMM(1, 1, 1, 1, 3),
    // A k-contiguous, B k-contiguous: T V^T
    TSR_GEMM(0, 0, 0, 1, 1), TSR_GEMM(0, 0, 0, 2, 2), TSR_GEMM(0, 0, 0, 3, 3),
};

hipError_t launch_gemm(const GemmLaunch& L, const GemmVariant& v, hipStream_t stream) {
    if (L.n_tiles <= 0) return hipSuccess;
    for (const Entry& e : kTable) {
        if (e.v.a_kstrided == v.a_kstrided && e.v.b_kstrided == v.b_kstrided && e.v.a_bf16 == v.a_bf16 &&
            e.v.a_pieces == v.a_pieces && e.v.b_pieces == v.b_pieces) {
            hipLaunchKernelGGL(e.fn, dim3(L.n_tiles), dim3(NTHREADS), 0, stream, L);
            return hipGetLastError();
        }
    }
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------ split-k reduction
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ReduceProblem* probs, const ReduceProblem single,
                                                            const float alpha, const float beta) {
    const ReduceProblem* p = probs ? probs + blockIdx.y : &single;
    const int M = p->M, N = p->N, splits = p->splits;
    const long long total = (long long)M * N;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (long long)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int k = 0; k < splits; ++k) s += p->part[(long long)k * p->stride + i];
        const long long o = (i / N) * p->ldc + (i % N);
        float v = alpha * s;
        if (beta != 0.0f) v += beta * p->out[o];
        p->out[o] = v;
    }
}

hipError_t launch_splitk_reduce(const ReduceProblem* probs_dev, const ReduceProblem* single, int count,
                                int max_elems, float alpha, float beta, hipStream_t stream) {
    if (count <= 0 || max_elems <= 0) return hipSuccess;
    int bx = (max_elems + 255) / 256;
    if (bx > 1024) bx = 1024;
    ReduceProblem s{};
    if (single) s = *single;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(bx, count), dim3(256), 0, stream, probs_dev, s, alpha, beta);
    return hipGetLastError();
}

}  // namespace tsr
