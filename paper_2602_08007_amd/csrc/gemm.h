// Grouped tall-skinny GEMM family on the gfx950 matrix cores (internal interface).
//
// One launch computes, for every tile in a tile list,
//     C[tile] = alpha * op(A) op(B) [tile] + beta * C[tile]          (fp32 output)
// with op(A) M x K and op(B) K x N taken from row-major storage in either orientation.
// Operands are fp32 (A may also be bf16); they are cut into 1..3 bf16 pieces and the
// leading cross products are accumulated in fp32 by v_mfma_f32_32x32x16_bf16.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsr {

struct GemmProblem {
    const void* A;      // k-contiguous: element (i,k) at A[i*lda + k]; k-strided: A[k*lda + i]
    const float* B;     // k-contiguous: element (j,k) at B[j*ldb + k]; k-strided: B[k*ldb + j]
    float* C;           // row-major M x N, leading dimension ldc
    long long lda, ldb, ldc;
    long long c_split_stride;  // elements between the partial outputs of consecutive k-splits
    int M, N, K;
    int kchunk;         // K range handled by one tile (multiple of 32); K if no split
};

struct GemmTile {       // one workgroup's work
    int prob, tm, tn, ks;
};

struct GemmLaunch {
    const GemmProblem* probs;  // device array (grouped) or nullptr
    const GemmTile* tiles;     // device array (grouped) or nullptr
    GemmProblem single;        // used when tiles == nullptr
    int tiles_m, tiles_n, ksplit;  // decode of blockIdx when tiles == nullptr
    int n_tiles;               // grid size
    float alpha, beta;         // epilogue scalars of the whole launch; beta == 0: C is not read
};

// Operand layout / precision of one instantiation.
struct GemmVariant {
    int a_kstrided;   // 0: A stored M x K (k contiguous), 1: A stored K x M
    int b_kstrided;   // 0: B stored N x K (k contiguous), 1: B stored K x N
    int a_bf16;       // A elements are bf16 (then a_pieces must be 1)
    int a_pieces;     // 1..3
    int b_pieces;     // 1..3
};

constexpr int GEMM_BM = 128;
constexpr int GEMM_BN = 128;

// Enqueue one grouped GEMM.  Returns hipSuccess or the launch error; an unsupported
// variant returns hipErrorInvalidValue.
hipError_t launch_gemm(const GemmLaunch& L, const GemmVariant& v, hipStream_t stream);

// out[i] = alpha * sum_{s<splits} part[s*stride + i] + beta * out[i], i over an M x N
// matrix with leading dimension ldc (partials are dense M x N).  Summed in split order.
struct ReduceProblem {
    const float* part; float* out;
    long long stride, ldc;
    int M, N, splits;
};
hipError_t launch_splitk_reduce(const ReduceProblem* probs_dev, const ReduceProblem* single,
                                int count, int max_elems, float alpha, float beta, hipStream_t stream);

}  // namespace tsr
