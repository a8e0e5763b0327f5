// bf16 x bf16 -> fp32 "NT" GEMM family for the bf16 step path (internal interface).
//
//   C[tile] = alpha * A B^T [tile] + beta * C[tile]
// A is M x K, B is N x K, both row-major with k contiguous (bf16; B may also be fp32 and is
// then rounded to bf16 on the way into LDS).  Output is fp32 (optionally into k-split
// partial buffers) or bf16.  All operands of the per-step path are brought into this one
// form (bf16 shadows of U, U^T, V, V^T; P^T and T as bf16 intermediates; D^T from the Adam
// kernel), so a single tuned kernel serves G V, U^T P, U D and the fused T V^T update.
#pragma once
#include <hip/hip_runtime.h>

#include "small.h"

namespace tsr {

struct NtProblem {
    const void* A;          // bf16, M x K, leading dimension lda
    const void* B;          // bf16 (or fp32), N x K, leading dimension ldb
    void* C;                // fp32 or bf16, M x N, leading dimension ldc
    long long lda, ldb, ldc;
    long long c_split_stride;
    int M, N, K;
    int kchunk;             // multiple of 64
    const AdamTBlock* adam; // fused Adam epilogue (NtVariant::fused_adam): this core's moment arrays
    long long b_piece_stride;   // NtVariant::b_pieces > 1: elements between the bf16 pieces of B
};

struct NtTile { int prob, tm, tn, ks; };     // prob < 0: idle workgroup
struct NtRange { int begin, end; };          // tiles [begin, end) of one persistent workgroup

// With `ranges` set the launch is persistent: workgroup w walks tiles[ranges[w].begin ..
// ranges[w].end) and keeps its load pipeline running across tile boundaries (the k-tiles of the
// next tile are on their way while the current tile finishes and is written out); n_tiles is
// then the number of workgroups.  The read-modify-write epilogue (beta != 0) has one persistent
// form only, NT_128x128_WS.
struct NtLaunch {
    const NtProblem* probs;
    const NtTile* tiles;
    const NtRange* ranges;
    int n_tiles;
    float alpha, beta;
    AdamScalars adam;       // fused Adam epilogue only
};

enum NtShape {
    NT_128x128 = 0,         // 64-deep k-tiles, two workgroups per compute unit
    NT_64x256 = 1,          // P^T of ranks up to 64
    NT_64x64 = 2,           // cores up to 256 x 256
    NT_128x128_K32 = 3,     // 32-deep k-tiles; with two pieces of B: the refresh products
    NT_256x128_K32 = 4,     // wide-tile kernel, two pieces of B only
    NT_256x256_K32 = 5,     // wide-tile kernel, one workgroup per compute unit
    NT_128x128_WS = 6,      // wave-specialised read-modify-write kernel: persistent launches (ranges) of fp32
                            // C = beta C + alpha A B^T with K == 512 in every problem, nothing else
    NT_SHAPES = 7
};
inline int nt_tile_m(int s) {
    static const int tm[NT_SHAPES] = {128, 64, 64, 128, 256, 256, 128};
    return tm[s];
}
inline int nt_tile_n(int s) {
    static const int tn[NT_SHAPES] = {128, 256, 64, 128, 128, 256, 128};
    return tn[s];
}

struct NtVariant {
    int shape;      // NtShape
    int b_f32;      // B operand stored as fp32
    int out_bf16;   // C stored as bf16 (beta ignored)
    int fused_adam; // persistent launches only: C (an r x r core, ldc = r) is final after this GEMM and
                    // the epilogue runs Adam on it (C, M, Vm, D and the bf16 D^T written there)
    int b_pieces;   // 0 or 1: B is one bf16 (or fp32) array; 2, 3: B is the sum of that many bf16 arrays
                    // (fp32 output, no read-modify-write, one tile per workgroup only)
};

hipError_t launch_nt_gemm(const NtLaunch& L, const NtVariant& v, hipStream_t stream);
int nt_wgs_per_cu(int shape);   // resident workgroups per CU the kernel of this shape is built for

// fp32 bases -> bf16 shadows: X (rows x r, contiguous fp32) -> Xb (rows x ldx bf16) and
// XTb (r x ldt bf16, the transpose); padding columns are written as zeros.  XFb (optional,
// r % 16 == 0) is the same matrix in MFMA-fragment order for the fused lift kernel: rows in
// groups of 32 (zero rows up to the next multiple of 32), and for group g and 16-wide k step s
// one contiguous 1 KiB record holding, for lane = 32 h + l, the 8 values X[32 g + l][16 s + 8 h ..].
// XTFb (optional, r % 32 == 0) is X^T in fragment order for the projection kernel: for the
// group g of 32 columns of X and the 16-wide step s over its rows one contiguous 1 KiB record
// holding, for lane = 32 h + l, the 8 values X[16 s + 8 h ..][32 g + l] (zeros beyond the last row).
struct ShadowBlock {
    const float* X; void* Xb; void* XTb; void* XFb; void* XTFb;
    int rows, r; long long ldx, ldt;
};
// Projection P^T = V^T G^T for one 128- or 64-row panel of a bf16 gradient per workgroup (r = 128
// or 256): the panel's accumulators (r x 128) stay in registers over the whole contraction, G goes
// through LDS, V^T comes straight from its fragment-order copy.  G == nullptr: idle workgroup.
struct ProjItem {
    const void* G;       // bf16 m x n, leading dimension ldg (16-byte aligned rows, n % 8 == 0)
    const void* VTf;     // ShadowBlock::XTFb of V
    void* PT;            // bf16 r x m, leading dimension ldp
    long long ldg, ldp;
    int m, n, row0;
};
bool proj_supports_rank(int r);
// depth: gradient tiles in flight per workgroup: 2 (two workgroups per compute unit) or 4 (one)
hipError_t launch_proj(const ProjItem* items_dev, int n_items, int r, int depth, hipStream_t stream);

// ---- operands of the refresh GEMMs in the k-contiguous bf16 form of this family
// Transposed bf16 copy of a gradient: dst (cols x rows, leading dimension ldd >= rows rounded up to 8,
// the padding written as zeros) = src^T for src (rows x cols bf16, leading dimension lds, even).
struct TransposeBlock {
    const void* src; void* dst;
    long long ld_src, ld_dst;
    int rows, cols;
};
hipError_t launch_transpose_bf16(const TransposeBlock* table_dev, int blocks, int max_rows, int max_cols, hipStream_t stream);

// An fp32 matrix X (rows x k, contiguous) as `pieces` bf16 matrices of its transpose: piece p
// (k rows of pitch ld_dst, at dst + p * piece_stride elements) holds the p-th term of
// x = x0 + x1 (+ x2) with x0 = bf16(x), x1 = bf16(x - x0), ...; columns rows .. up to the next
// multiple of 8 are written as zeros, nothing beyond (pieces may sit side by side in one row).
struct SplitBlock {
    const float* X; void* dst;
    long long ld_dst, piece_stride;
    int rows, k;
};
hipError_t launch_split_transpose(const SplitBlock* table_dev, int blocks, int max_rows, int max_k, int pieces,
                                  hipStream_t stream);
// The same pieces without the transposition: piece p (rows of pitch ld_dst, at dst + p * piece_stride) of
// X (rows x k, contiguous); columns k .. up to the next multiple of 8 are written as zeros.
hipError_t launch_split_rows(const SplitBlock* table_dev, int blocks, int max_rows, int max_k, int pieces, hipStream_t stream);

hipError_t launch_shadows(const ShadowBlock* table_dev, int blocks, int max_rows, int max_r, hipStream_t stream);

}  // namespace tsr
