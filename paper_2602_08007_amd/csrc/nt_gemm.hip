// bf16 NT GEMMs for the per-step path and the refresh on gfx950: C = alpha A B^T + beta C with A (M x K)
// and B (N x K) both k-contiguous, v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  Four kernels:
//   nt_gemm_kernel             128 x 128 (and smaller) tiles, 256 threads, two register stages + two LDS
//                              buffers; stores, bf16 stores or a read-modify-write epilogue; B in pieces
//   nt_wide_kernel             256 x 256 / 256 x 128 tiles, one workgroup per compute unit, hand-scheduled
//   nt_gemm_persistent_kernel  a workgroup walks a list of tiles, optionally with Adam in the epilogue
//   nt_rmw_ws_kernel           the weight update at rank 512: separate waves for MFMAs, operands and C
// and the projection kernel (a whole P^T panel in accumulators), the bf16 shadows of the bases and the
// operand preparation of the refresh products.
#include "nt_gemm.h"

namespace tsr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int NT_THREADS = 256;
// LDS rows are padded by 8 bf16 (16 bytes): 80-byte rows for 32-deep k-tiles, 144-byte rows
// for 64-deep ones; both give conflict-free 16-byte fragment reads.

template <int CH, bool F32> struct NtStage;      // CH = 16-byte chunks per thread
template <int CH> struct NtStage<CH, false> { u32x4 v[CH]; };
template <int CH> struct NtStage<CH, true> { f32x4 v[CH][2]; };

// Raw buffer loads: one descriptor (SGPRs) per operand, a 32-bit per-lane byte offset.  A
// per-lane offset at or beyond the descriptor's size reads as zero, which is the row guard
// (rows beyond the operand lie beyond its last byte); the k guard of the last, partial k-tile
// is a mask applied to the loaded words.  No branches, no 64-bit address arithmetic.
typedef __amdgpu_buffer_rsrc_t nt_rsrc_t;
__device__ inline nt_rsrc_t nt_make_rsrc(const void* p, long long bytes) {
    const int n = (bytes > 0x7fffffffLL) ? 0x7fffffff : (int)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), (short)0, n, 0x00020000);
}

// The same from values that are equal in every lane but that the compiler cannot prove so (loaded after
// the kernel's own global stores): taken from the first lane, so that the descriptor lives in SGPRs.
__device__ inline int nt_uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ inline nt_rsrc_t nt_make_rsrc_uni(const void* p, long long bytes) {
    const unsigned long long a = (unsigned long long)p;
    const unsigned lo = (unsigned)nt_uni((int)(unsigned)a), hi = (unsigned)nt_uni((int)(unsigned)(a >> 32));
    const int n = nt_uni((bytes > 0x7fffffffLL) ? 0x7fffffff : (int)bytes);
    return __builtin_amdgcn_make_buffer_rsrc((void*)(((unsigned long long)hi << 32) | lo), (short)0, n, 0x00020000);
}

// Launch tables (written by the host before the launch, never by a kernel) read through the constant
// address space: with a wave-uniform index these are scalar loads, which have a counter of their own
// and do not wait for the vector loads in flight.
#define NT_CONST __attribute__((address_space(4)))
template <typename T> __device__ inline const NT_CONST T* nt_const(const T* p) { return (const NT_CONST T*)p; }

// rows x K operand, k contiguous; tile rows row0.., k0..k0+BK-1.  Thread t owns chunks
// c = t + 256*it: row c/(BK/8), k offset (c%(BK/8))*8 (the same k offset for every chunk of a
// thread, since 256 is a multiple of BK/8).  `live` = false (wave-uniform): the whole tile reads
// as zero without touching memory (poisoned offsets), which lets the pipeline issue its loads
// unconditionally.  The k guard of a partial last k-tile is applied by nt_store.
template <int ROWS, int BK, bool F32>
__device__ inline void nt_load(NtStage<ROWS * BK / 8 / NT_THREADS, F32>& s, nt_rsrc_t rs, unsigned ld_bytes, int row0,
                               int k0, bool live, int tid) {
    constexpr int CPR = BK / 8;
    constexpr int ESZ = F32 ? 4 : 2;
    constexpr int CH = ROWS * CPR / NT_THREADS;
    const unsigned poison = live ? 0u : 0x80000000u;       // in-range offsets stay below 2^31 (checked on the host)
#pragma unroll
    for (int it = 0; it < CH; ++it) {
        const int c = tid + NT_THREADS * it;
        const unsigned grow = row0 + c / CPR;
        const int gk = k0 + (c % CPR) * 8;
        const unsigned voff = (grow * ld_bytes + (unsigned)gk * ESZ) | poison;
        if constexpr (F32) {
            s.v[it][0] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, 0, 0));
            s.v[it][1] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, 16, 0));
        } else {
            s.v[it] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, 0, 0));
        }
    }
}

// Stage -> LDS.  `valid` = elements of this thread's chunks that lie before the end of the k range
// (8 or more: all of them; only the last k-tile of a range has fewer); the rest is stored as zero.
template <int ROWS, int BK, bool F32>
__device__ inline void nt_store(const NtStage<ROWS * BK / 8 / NT_THREADS, F32>& s, unsigned short* lds, int tid, int valid,
                                bool tail) {
    constexpr int CPR = BK / 8, KP = BK + 8;
    if (!tail) {                                            // wave-uniform: every k-tile but the last of a range
#pragma unroll
        for (int it = 0; it < ROWS * CPR / NT_THREADS; ++it) {
            const int c = tid + NT_THREADS * it;
            unsigned short* dst = lds + (c / CPR) * KP + (c % CPR) * 8;
            if constexpr (F32) {
                bf16x8 h;
#pragma unroll
                for (int j = 0; j < 8; ++j) h[j] = (__bf16)s.v[it][j >> 2][j & 3];
                *(bf16x8*)dst = h;
            } else {
                *(u32x4*)dst = s.v[it];
            }
        }
        return;
    }
    u32x4 m;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        m[j] = ((2 * j < valid) ? 0x0000ffffu : 0u) | ((2 * j + 1 < valid) ? 0xffff0000u : 0u);
#pragma unroll
    for (int it = 0; it < ROWS * CPR / NT_THREADS; ++it) {
        const int c = tid + NT_THREADS * it;
        unsigned short* dst = lds + (c / CPR) * KP + (c % CPR) * 8;
        if constexpr (F32) {
            bf16x8 h;
#pragma unroll
            for (int j = 0; j < 8; ++j) h[j] = (__bf16)s.v[it][j >> 2][j & 3];
            *(u32x4*)dst = __builtin_bit_cast(u32x4, h) & m;
        } else {
            *(u32x4*)dst = s.v[it] & m;
        }
    }
}

__device__ inline unsigned short f32_to_bf16_bits(float f) {
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(unsigned short, h);
}

// OUT: 0 = fp32 store (alpha only), 1 = bf16 store (alpha only), 2 = fp32 read-modify-write
// NP: B is the sum of NP bf16 arrays of the same shape (an fp32 operand cut into pieces, piece p at
// B + p * b_piece_stride elements, smallest piece last): every A fragment meets the fragments of
// all pieces, so the product carries the fp32-grade operand at NP MFMAs per tile product while A is
// staged and read once.
template <int TM, int TN, int WM, int WN, int NT_BK, bool B_F32, int OUT, int MINB, int NP = 1>
__global__ __launch_bounds__(NT_THREADS, MINB) void nt_gemm_kernel(const NtLaunch L) {
    constexpr bool OUT_BF16 = (OUT == 1);
    constexpr bool RMW = (OUT == 2);
    static_assert(WM * WN == 4, "four waves");
    constexpr int NT_KP = NT_BK + 8;
    constexpr int FM = TM / WM / 32, FN = TN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
    constexpr int A_ELEMS = TM * NT_KP, B_ELEMS = TN * NT_KP, BUF = A_ELEMS + NP * B_ELEMS;
    static_assert(NP == 1 || !B_F32, "pieces are bf16");

    const NtTile t = L.tiles[blockIdx.x];
    if (t.prob < 0) return;
    const NtProblem* pp = L.probs + t.prob;
    const void* A = pp->A;
    const void* B = pp->B;
    const long long lda = pp->lda, ldb = pp->ldb, ldc = pp->ldc;
    const int M = pp->M, N = pp->N, K = pp->K;
    const float alpha = L.alpha, beta = L.beta;
    const int kbeg = t.ks * pp->kchunk;
    const int kend = min(K, kbeg + pp->kchunk);
    const int row0 = t.tm * TM, col0 = t.tn * TN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // Operands have 16-byte aligned bases and rows, and K rounded up to 8 elements still lies
    // inside every row (the host routes anything else to the generic kernels): a 16-byte chunk is
    // then either wholly inside the operand's extent or wholly outside it.
    const long long k8 = (K + 7) & ~7;
    const nt_rsrc_t rA = nt_make_rsrc(A, ((long long)(M - 1) * lda + k8) * 2);
    nt_rsrc_t rB[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p)
        rB[p] = nt_make_rsrc((const char*)B + (long long)p * pp->b_piece_stride * 2, ((long long)(N - 1) * ldb + k8) * (B_F32 ? 4 : 2));
    const unsigned lda_b = (unsigned)lda * 2u, ldb_b = (unsigned)ldb * (B_F32 ? 4u : 2u);

    // For the read-modify-write epilogue the C tile is fetched into registers before the last two
    // k-tiles are multiplied (see the loop): by then the second register stage has nothing left to
    // prefetch, so the tile takes its registers, and the k-loop keeps both stages up to that point.
    f32x16 cold[RMW ? FM : 1][RMW ? FN : 1];
    const float out_scale = alpha;
    const bool skip_products = RMW && alpha == 0.0f;
    // output descriptor: guards poison the per-lane offset (the wave-uniform offset is not
    // range-checked by the hardware)
    constexpr int CSZ = OUT_BF16 ? 2 : 4;
    const nt_rsrc_t rC = nt_make_rsrc((const char*)pp->C + (long long)t.ks * pp->c_split_stride * CSZ,
                                      ((long long)(M - 1) * ldc + N) * CSZ);
    const unsigned ldc_b = (unsigned)ldc * CSZ;
    auto c_voff = [&](int i, int j, int e) -> unsigned {
        const int col = col0 + wn * (FN * 32) + j * 32 + (lane & 31);
        const int row = row0 + wm * (FM * 32) + i * 32 + (lane >> 5) * 4 + (e >> 2) * 8 + (e & 3);
        return (row < M && col < N) ? (unsigned)row * ldc_b + (unsigned)col * CSZ : 0x80000000u;
    };
    auto load_c = [&]() {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    cold[i][j][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rC, (int)c_voff(i, j, e), 0, 0));
    };
    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Two k-tiles travel in registers ahead of the one being multiplied (ring of two register
    // stages), one more sits in the other LDS buffer: global latency hides behind two k-tiles of
    // MFMAs per workgroup.
    constexpr int NSTAGE = 2;
    NtStage<TM * NT_BK / 8 / NT_THREADS, false> stA[NSTAGE];
    NtStage<TN * NT_BK / 8 / NT_THREADS, B_F32> stB[NSTAGE][NP];
    const int nk = (kend > kbeg && !skip_products) ? (kend - kbeg + NT_BK - 1) / NT_BK : 0;

    // Loads are issued for every slot of the pipeline whether or not the k range still has a tile for
    // it (tiles at or beyond nk read as zero without a memory access), and every stage is stored: the
    // loop body is then free of branches around memory instructions, and the waits the compiler
    // places before a stage is stored let the younger stage's loads stay in flight.
    const int k_in_tile = (tid % (NT_BK / 8)) * 8;          // k offset of this thread's chunks within a k-tile
    auto load = [&](int slot, int tile) {
        const int k0 = kbeg + tile * NT_BK;
        const bool live = tile < nk;
        nt_load<TM, NT_BK, false>(stA[slot], rA, lda_b, row0, k0, live, tid);
#pragma unroll
        for (int p = 0; p < NP; ++p) nt_load<TN, NT_BK, B_F32>(stB[slot][p], rB[p], ldb_b, col0, k0, live, tid);
    };
    auto store = [&](int slot, int buf, int tile) {
        unsigned short* d = lds + buf * BUF;
        const int k0 = kbeg + tile * NT_BK;
        const bool tail = k0 + NT_BK > kend;
        nt_store<TM, NT_BK, false>(stA[slot], d, tid, kend - (k0 + k_in_tile), tail);
#pragma unroll
        for (int p = 0; p < NP; ++p)
            nt_store<TN, NT_BK, B_F32>(stB[slot][p], d + A_ELEMS + p * B_ELEMS, tid, kend - (k0 + k_in_tile), tail);
    };
    auto compute = [&](int buf) {
        const unsigned short* sA = lds + buf * BUF;
        const unsigned short* sB = sA + A_ELEMS;
#pragma unroll
        for (int kk = 0; kk < NT_BK / 16; ++kk) {
            const int kofs = kk * 16 + (lane >> 5) * 8;
            bf16x8 fa[FM], fb[NP][FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                fa[i] = *(const bf16x8*)(sA + (wm * (FM * 32) + i * 32 + (lane & 31)) * NT_KP + kofs);
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    fb[p][j] = *(const bf16x8*)(sB + p * B_ELEMS + (wn * (FN * 32) + j * 32 + (lane & 31)) * NT_KP + kofs);
#pragma unroll
            for (int p = NP - 1; p >= 0; --p)               // smallest piece first
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[p][j], acc[i][j], 0, 0, 0);
        }
    };

    if (nk > 0) {
        if constexpr (NSTAGE == 2) {
            // prologue: tile 0 -> LDS buffer 0; tiles 1 and 2 -> register stages 1 and 0
            load(0, 0);
            store(0, 0, 0);
            __syncthreads();
            load(1, 1);
            __builtin_amdgcn_sched_barrier(0);               // keep the issue order: the loop waits for the older stage only
            load(0, 2);
            // the pair (it, it + 1): multiply LDS buffer 0, move tile it + 1 (stage 1) into buffer 1 and
            // refill that stage with tile it + 3; then the same with the roles exchanged.  With an odd
            // nk the last half-step multiplies a tile of zeros.
            if constexpr (!RMW) {
                for (int it = 0; it < nk; it += 2) {
                    compute(0);
                    store(1, 1, it + 1);
                    __syncthreads();
                    load(1, it + 3);
                    compute(1);
                    store(0, 0, it + 2);
                    __syncthreads();
                    load(0, it + 4);
                }
            } else {
                // the last pair is peeled: no loads any more (stage 0 is dead), the C tile is fetched instead
                int it = 0;
                for (; it + 2 < nk; it += 2) {
                    compute(0);
                    store(1, 1, it + 1);
                    __syncthreads();
                    load(1, it + 3);
                    compute(1);
                    store(0, 0, it + 2);
                    __syncthreads();
                    load(0, it + 4);
                }
                __builtin_amdgcn_sched_barrier(0);
                compute(0);
                store(1, 1, it + 1);
                __builtin_amdgcn_sched_barrier(0);
                load_c();
                __syncthreads();
                compute(1);
            }
        }
    } else if constexpr (RMW) {
        load_c();
    }

    // epilogue: lane holds column (lane & 31); rows 8*(e/4) + 4*(lane>>5) + e%4 of each 32x32 tile
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const unsigned vo = c_voff(i, j, e);
                if constexpr (OUT_BF16) {
                    __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16_bits(out_scale * acc[i][j][e]), rC, (int)vo, 0, 0);
                } else {
                    float v = out_scale * acc[i][j][e];
                    if constexpr (RMW) v += beta * cold[i][j][e];
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rC, (int)vo, 0, 0);
                }
            }
}

// ------------------------------------------------------------------ wide-tile variant
// One workgroup per compute unit, four waves in a 2 x 2 layout, each wave FM x FN fragments of
// 32 x 32 (256 x 256 outputs per workgroup with FM = FN = 4), 32-deep k-tiles.  A tile twice as
// wide as the 128 x 128 kernels' halves the operand traffic per flop, but leaves one wave per SIMD,
// so nothing hides a wave's own latencies unless its instruction stream does; and a wave that issues
// a block of LDS stores or of global loads issues no MFMA until the block has drained (a probe of
// this loop without global memory: MFMAs alone 2.16 PFLOP/s; with the eight stage stores of a
// k-tile issued as a block 1.6; spread over the MFMAs 1.94; in the unpadded, XOR-swizzled LDS
// layout below 2.05).  The loop is therefore scheduled by hand (scheduling barriers pin the order):
//   k step 0: MFMAs from F[0]; the fragments of k step 1 are read under the first half, the next
//             k-tile moves from its register stage into the other LDS buffer under the second half,
//             one or two stores per MFMA pair;
//   k step 1: MFMAs from F[1]; the barrier after the first quarter; then the loads of the k-tile
//             three ahead and the first fragments of the next k-tile, again a few per MFMA pair.
// LDS rows are 64 bytes (four 16-byte chunks), unpadded; chunk c of row r sits at position
// c ^ ((r >> 1) & 3): fragment reads and stage stores are both free of bank conflicts.
// OUT: 0 = fp32 store, 1 = bf16 store.  NP: pieces of B (see nt_gemm_kernel).
template <int FM, int FN, int NP, int OUT>
__global__ __launch_bounds__(NT_THREADS, 1) void nt_wide_kernel(const NtLaunch L) {
    constexpr bool OUT_BF16 = (OUT == 1);
    constexpr int BK = 32;
    constexpr int TM = 2 * FM * 32, TN = 2 * FN * 32;
    constexpr int A_ELEMS = TM * BK, B_ELEMS = TN * BK, BUF = A_ELEMS + NP * B_ELEMS;
    constexpr int CHA = TM * BK / 8 / NT_THREADS, CHB = TN * BK / 8 / NT_THREADS;
    constexpr int CH = CHA + NP * CHB;                      // 16-byte chunks per thread and k-tile
    constexpr int NFRAG = FM + NP * FN;                     // fragment reads per k step
    constexpr int NMFMA = FM * FN * NP;                     // MFMAs per k step
    static_assert(NMFMA % 8 == 0 && NFRAG % 4 == 0 && CH % 4 == 0, "the schedule issues the MFMAs of a k step in eight groups");
    constexpr int GRP = NMFMA / 8;
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];

    const NtTile t = L.tiles[blockIdx.x];
    if (t.prob < 0) return;
    const NtProblem* pp = L.probs + t.prob;
    const int M = pp->M, N = pp->N, K = pp->K;
    const long long lda = pp->lda, ldb = pp->ldb, ldc = pp->ldc;
    const int kbeg = t.ks * pp->kchunk;
    const int kend = min(K, kbeg + pp->kchunk);
    const int row0 = t.tm * TM, col0 = t.tn * TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const long long k8 = (K + 7) & ~7;
    const nt_rsrc_t rA = nt_make_rsrc(pp->A, ((long long)(M - 1) * lda + k8) * 2);
    nt_rsrc_t rB[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p)
        rB[p] = nt_make_rsrc((const char*)pp->B + (long long)p * pp->b_piece_stride * 2, ((long long)(N - 1) * ldb + k8) * 2);
    const unsigned lda_b = (unsigned)lda * 2u, ldb_b = (unsigned)ldb * 2u;
    const int nk = (kend > kbeg) ? (kend - kbeg + BK - 1) / BK : 0;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Chunk x of a thread (x < CHA: operand A, else piece (x - CHA) / CHB of B): row (tid + 256 u) / 4
    // of the operand's tile, k offset (tid % 4) * 8 (the same for all chunks of a thread).
    u32x4 st[2][CH];
    const int k_in_tile = (tid & 3) * 8;
    const int swz_row = tid >> 2;                            // row of chunk u = swz_row + 64 u
    auto load_chunk = [&](int slot, int tile, int x) {      // unconditional: tiles at or beyond nk read as zero
        const unsigned poison = (tile < nk) ? 0u : 0x80000000u;
        const int k0 = kbeg + tile * BK + k_in_tile;
        if (x < CHA) {
            const unsigned voff = ((unsigned)(row0 + swz_row + 64 * x) * lda_b + (unsigned)k0 * 2u) | poison;
            st[slot][x] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rA, (int)voff, 0, 0));
        } else {
            const int p = (x - CHA) / CHB, u = (x - CHA) % CHB;
            const unsigned voff = ((unsigned)(col0 + swz_row + 64 * u) * ldb_b + (unsigned)k0 * 2u) | poison;
            st[slot][x] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rB[p], (int)voff, 0, 0));
        }
    };
    // k guard of a stage: all ones, or the mask of the elements before kend in the last k-tile of the range
    auto tail_mask = [&](int tile) -> u32x4 {
        const int valid = kend - (kbeg + tile * BK + k_in_tile);
        u32x4 m;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            m[j] = ((2 * j < valid) ? 0x0000ffffu : 0u) | ((2 * j + 1 < valid) ? 0xffff0000u : 0u);
        return m;
    };
    auto store_chunk = [&](int slot, int buf, int x, u32x4 m) {
        int base, u;
        if (x < CHA) { base = 0; u = x; }
        else { base = A_ELEMS + ((x - CHA) / CHB) * B_ELEMS; u = (x - CHA) % CHB; }
        const int r = swz_row + 64 * u;
        const int pos = (tid & 3) ^ ((r >> 1) & 3);
        *(u32x4*)(lds + buf * BUF + base + r * BK + pos * 8) = st[slot][x] & m;
    };
    // fragment f of k step kk of LDS buffer buf: f < FM: A rows; else piece (f - FM) / FN, column group (f - FM) % FN
    const int l32 = lane & 31, h = lane >> 5;
    auto frag = [&](int buf, int kk, int f) -> bf16x8 {
        int base, r;
        if (f < FM) { base = 0; r = wm * (FM * 32) + f * 32 + l32; }
        else { const int g = f - FM; base = A_ELEMS + (g / FN) * B_ELEMS; r = wn * (FN * 32) + (g % FN) * 32 + l32; }
        const int pos = (kk * 2 + h) ^ ((r >> 1) & 3);
        return *(const bf16x8*)(lds + buf * BUF + base + r * BK + pos * 8);
    };
    bf16x8 F[2][NFRAG];
    // MFMA number q of a k step: pieces from the smallest to the largest, then rows, then columns
    auto mfma = [&](const bf16x8* f, int q) {
        const int p = NP - 1 - q / (FM * FN), i = (q / FN) % FM, j = q % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], f[FM + p * FN + j], acc[i][j], 0, 0, 0);
    };
#define NT_SB __builtin_amdgcn_sched_barrier(0)

    if (nk > 0) {
#pragma unroll
        for (int x = 0; x < CH; ++x) load_chunk(0, 0, x);
        {
            const u32x4 m = tail_mask(0);
#pragma unroll
            for (int x = 0; x < CH; ++x) store_chunk(0, 0, x, m);
        }
        __syncthreads();
#pragma unroll
        for (int x = 0; x < CH; ++x) load_chunk(1, 1, x);
        NT_SB;                                               // keep the issue order: the loop waits for the older stage only
#pragma unroll
        for (int x = 0; x < CH; ++x) load_chunk(0, 2, x);
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) F[0][f] = frag(0, 0, f);
        // tile `it` sits in LDS buffer it & 1, tile it + 1 in register stage (it + 1) & 1, tile it + 2 in
        // the other stage; F[0] holds the fragments of k step 0 of tile `it`
        auto step = [&](int cur, int it) {
            const int oth = cur ^ 1;
            const u32x4 m = tail_mask(it + 1);
            // ---- k step 0
            NT_SB;
#pragma unroll
            for (int g = 0; g < 8; ++g) {
#pragma unroll
                for (int u = 0; u < GRP; ++u) mfma(F[0], g * GRP + u);
                NT_SB;
                if (g < 4) {
#pragma unroll
                    for (int f = g * NFRAG / 4; f < (g + 1) * NFRAG / 4; ++f) F[1][f] = frag(cur, 1, f);
                } else {                                      // register stage (it + 1) & 1 == oth -> LDS buffer oth
#pragma unroll
                    for (int x = (g - 4) * CH / 4; x < (g - 3) * CH / 4; ++x) store_chunk(oth, oth, x, m);
                }
                NT_SB;
            }
            // ---- k step 1
#pragma unroll
            for (int u = 0; u < 2 * GRP; ++u) mfma(F[1], u);
            NT_SB;
            __syncthreads();
            NT_SB;
#pragma unroll
            for (int g = 2; g < 8; ++g) {
#pragma unroll
                for (int x = (g - 2) * CH / 6; x < (g - 1) * CH / 6; ++x) load_chunk(oth, it + 3, x);
#pragma unroll
                for (int u = 0; u < GRP; ++u) mfma(F[1], g * GRP + u);
                NT_SB;
                if (g < 6) {
#pragma unroll
                    for (int f = (g - 2) * NFRAG / 4; f < (g - 1) * NFRAG / 4; ++f) F[0][f] = frag(oth, 0, f);
                    NT_SB;
                }
            }
        };
        for (int it = 0; it < nk; it += 2) {
            step(0, it);
            step(1, it + 1);                                  // with an odd nk: a tile of zeros
        }
    }
#undef NT_SB

    constexpr int CSZ = OUT_BF16 ? 2 : 4;
    const nt_rsrc_t rC = nt_make_rsrc((const char*)pp->C + (long long)t.ks * pp->c_split_stride * CSZ,
                                      ((long long)(M - 1) * ldc + N) * CSZ);
    const unsigned ldc_b = (unsigned)ldc * CSZ;
    const float alpha = L.alpha;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int col = col0 + wn * (FN * 32) + j * 32 + (lane & 31);
                const int row = row0 + wm * (FM * 32) + i * 32 + (lane >> 5) * 4 + (e >> 2) * 8 + (e & 3);
                const unsigned vo = (row < M && col < N) ? (unsigned)row * ldc_b + (unsigned)col * CSZ : 0x80000000u;
                if constexpr (OUT_BF16)
                    __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16_bits(alpha * acc[i][j][e]), rC, (int)vo, 0, 0);
                else
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, alpha * acc[i][j][e]), rC, (int)vo, 0, 0);
            }
}

// ------------------------------------------------------------------ persistent variant
// One workgroup walks a list of tiles.  The k-tiles of all its tiles form one stream that runs
// through the same pipeline as above (two register stages, two LDS buffers) without draining at
// tile boundaries: the loader cursor runs three k-tiles ahead of the compute cursor and moves on
// to the next tile by itself.  A tile's accumulators are written out when the compute cursor
// leaves it.  OUT: 0 = fp32 store, 1 = bf16 store, 3 = fp32 store of a core followed by Adam on it.
template <int TM, int TN, int WM, int WN, int NT_BK, bool B_F32, int OUT, int MINB>
__global__ __launch_bounds__(NT_THREADS, MINB) void nt_gemm_persistent_kernel(const NtLaunch L) {
    constexpr bool OUT_BF16 = (OUT == 1);
    static_assert(WM * WN == 4, "four waves");
    static_assert(OUT == 0 || OUT == 1 || OUT == 3, "no read-modify-write epilogue here");
    constexpr int NT_KP = NT_BK + 8;
    constexpr int FM = TM / WM / 32, FN = TN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
    constexpr int A_ELEMS = TM * NT_KP, B_ELEMS = TN * NT_KP, BUF = A_ELEMS + B_ELEMS;

    const NtRange range = L.ranges[blockIdx.x];
    if (range.begin >= range.end) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const float alpha = L.alpha;

    auto tile_nk = [&](const NtTile& t) -> int {
        const NtProblem* pp = L.probs + t.prob;
        const int kbeg = t.ks * pp->kchunk;
        const int kend = min(pp->K, kbeg + pp->kchunk);
        return (kend - kbeg + NT_BK - 1) / NT_BK;
    };
    int total = 0;                                           // k-tiles of the whole list
    for (int t = range.begin; t < range.end; ++t) total += tile_nk(L.tiles[t]);

    // ---- loader cursor
    int lt = range.begin, lk = 0;
    nt_rsrc_t rA, rB;
    unsigned lda_b, ldb_b;
    int l_row0, l_col0, l_kbeg, l_kend, l_nk;
    auto open_tile = [&](int t) {
        const NtTile tl = L.tiles[t];
        const NtProblem* pp = L.probs + tl.prob;
        const long long k8 = (pp->K + 7) & ~7;
        rA = nt_make_rsrc(pp->A, ((long long)(pp->M - 1) * pp->lda + k8) * 2);
        rB = nt_make_rsrc(pp->B, ((long long)(pp->N - 1) * pp->ldb + k8) * (B_F32 ? 4 : 2));
        lda_b = (unsigned)pp->lda * 2u;
        ldb_b = (unsigned)pp->ldb * (B_F32 ? 4u : 2u);
        l_row0 = tl.tm * TM; l_col0 = tl.tn * TN;
        l_kbeg = tl.ks * pp->kchunk;
        l_kend = min(pp->K, l_kbeg + pp->kchunk);
        l_nk = (l_kend - l_kbeg + NT_BK - 1) / NT_BK;
    };
    open_tile(lt);
    NtStage<TM * NT_BK / 8 / NT_THREADS, false> stA[2];
    NtStage<TN * NT_BK / 8 / NT_THREADS, B_F32> stB[2];
    // Loads are unconditional (beyond the end of the list they read as zero without a memory access)
    // and every stage is stored, so that the loop has no branch around a load: the compiler's waits
    // before a stage is stored then leave the younger stage's loads in flight.
    const int k_in_tile = (tid % (NT_BK / 8)) * 8;
    int st_valid[2] = {0, 0};                                // per stage: elements before the end of its k range
    bool st_tail[2] = {true, true};
    auto load_next = [&](int slot) {
        const bool live = lt < range.end;
        const int k0 = l_kbeg + lk * NT_BK;
        st_tail[slot] = !live || k0 + NT_BK > l_kend;
        st_valid[slot] = live ? l_kend - (k0 + k_in_tile) : 0;
        nt_load<TM, NT_BK, false>(stA[slot], rA, lda_b, l_row0, k0, live, tid);
        nt_load<TN, NT_BK, B_F32>(stB[slot], rB, ldb_b, l_col0, k0, live, tid);
        if (live && ++lk == l_nk) { lk = 0; if (++lt < range.end) open_tile(lt); }
    };
    auto store = [&](int slot, int buf) {
        unsigned short* d = lds + buf * BUF;
        nt_store<TM, NT_BK, false>(stA[slot], d, tid, st_valid[slot], st_tail[slot]);
        nt_store<TN, NT_BK, B_F32>(stB[slot], d + A_ELEMS, tid, st_valid[slot], st_tail[slot]);
    };

    // ---- compute cursor
    f32x16 acc[FM][FN];
    auto zero_acc = [&]() {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    };
    zero_acc();
    int ct = range.begin, ck = 0, c_nk = l_nk;
    auto compute = [&](int buf) {
        const unsigned short* sA = lds + buf * BUF;
        const unsigned short* sB = sA + A_ELEMS;
#pragma unroll
        for (int kk = 0; kk < NT_BK / 16; ++kk) {
            const int kofs = kk * 16 + (lane >> 5) * 8;
            bf16x8 fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                fa[i] = *(const bf16x8*)(sA + (wm * (FM * 32) + i * 32 + (lane & 31)) * NT_KP + kofs);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                fb[j] = *(const bf16x8*)(sB + (wn * (FN * 32) + j * 32 + (lane & 31)) * NT_KP + kofs);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };
    // after the last k-tile of a tile: write it out, start the next one
    auto finish_step = [&]() {
        if (++ck < c_nk) return;
        const NtTile t = L.tiles[ct];
        const NtProblem* pp = L.probs + t.prob;
        const int M = pp->M, N = pp->N;
        constexpr int CSZ = OUT_BF16 ? 2 : 4;
        const nt_rsrc_t rC = nt_make_rsrc((const char*)pp->C + (long long)t.ks * pp->c_split_stride * CSZ,
                                          ((long long)(M - 1) * pp->ldc + N) * CSZ);
        const unsigned ldc_b = (unsigned)pp->ldc * CSZ;
        const int row0 = t.tm * TM, col0 = t.tn * TN;
        AdamTBlock ab = {};
        const AdamScalars sc = L.adam;
        unsigned short dq[4] = {0, 0, 0, 0};
        if constexpr (OUT == 3) ab = *pp->adam;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int col = col0 + wn * (FN * 32) + j * 32 + (lane & 31);
                    const int row = row0 + wm * (FM * 32) + i * 32 + (lane >> 5) * 4 + (e >> 2) * 8 + (e & 3);
                    const unsigned vo = (row < M && col < N) ? (unsigned)row * ldc_b + (unsigned)col * CSZ : 0x80000000u;
                    if constexpr (OUT_BF16) {
                        __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16_bits(alpha * acc[i][j][e]), rC, (int)vo, 0, 0);
                    } else {
                        const float cv = alpha * acc[i][j][e];
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, cv), rC, (int)vo, 0, 0);
                        if constexpr (OUT == 3) {
                            // Adam on the finished core entry (Algorithm 1: moments, bias correction, D)
                            float d = 0.0f;
                            if (row < M && col < N) {
                                const long long idx = (long long)row * ab.r + col;
                                const float mm = sc.beta1 * ab.M[idx] + (1.0f - sc.beta1) * cv;
                                const float vv = sc.beta2 * ab.Vm[idx] + (1.0f - sc.beta2) * (cv * cv);
                                ab.M[idx] = mm;
                                ab.Vm[idx] = vv;
                                d = (mm * sc.inv_c1) / (sqrtf(vv * sc.inv_c2) + sc.eps);
                                ab.D[idx] = d;
                                if (!ab.DTf) ((unsigned short*)ab.DTb)[(long long)col * ab.ldt + row] = f32_to_bf16_bits(d);
                                if (ab.Db) ((unsigned short*)ab.Db)[(long long)row * ab.ldt + col] = f32_to_bf16_bits(d);
                            }
                            dq[e & 3] = f32_to_bf16_bits(d);
                            // D^T in fragment order: the four rows e & 3 = 0..3 of this lane are four
                            // neighbouring bf16 of one record (r % 32 == 0, so they are all inside D)
                            if ((e & 3) == 3 && ab.DTf && row < M && col < N) {
                                const int rw = row - 3;
                                const int ksteps = ab.r / 16;
                                uint2 pk;
                                pk.x = dq[0] | ((unsigned)dq[1] << 16);
                                pk.y = dq[2] | ((unsigned)dq[3] << 16);
                                *(uint2*)((unsigned short*)ab.DTf + (((long long)(col / 32) * ksteps + rw / 16) * 64 +
                                                                     ((rw % 16) / 8) * 32 + col % 32) * 8 + rw % 8) = pk;
                            }
                        }
                    }
                }
        zero_acc();
        ck = 0;
        if (++ct < range.end) c_nk = tile_nk(L.tiles[ct]);
    };

    // ---- the stream: step g multiplies LDS buffer g&1, moves step g+1 (register stage (g+1)&1)
    // into the other buffer and refills that stage with step g+3
    load_next(0);
    store(0, 0);
    __syncthreads();
    load_next(1);
    __builtin_amdgcn_sched_barrier(0);                       // keep the issue order: the loop waits for the older stage only
    load_next(0);
    for (int g = 0; g < total; g += 2) {
        compute(0);
        finish_step();
        store(1, 1);
        __syncthreads();
        load_next(1);
        if (g + 1 < total) {                                 // no memory instruction of the pipeline depends on this branch
            compute(1);
            finish_step();
        }
        store(0, 0);
        __syncthreads();
        load_next(0);
    }
}

typedef void (*nt_fn)(const NtLaunch);

// ------------------------------------------------------------------ wave-specialised read-modify-write kernel
// C = beta C + alpha A B^T by 128 x 128 tiles for a weight matrix C that streams from and to HBM while
// A and B come out of the L2.  A wave's vector-memory results return in the order the wave asked for
// them, so a wave that mixes the HBM stream with the operand loads waits for HBM latency at every
// operand tile.  Here each stream has waves of its own (twelve waves as launched, three per SIMD, one
// workgroup per compute unit, every wave passes the same barriers):
//   4 waves    multiply: fragments from LDS, MFMAs, the finished 128 x 128 accumulator tile goes to an
//              fp32 staging tile in LDS and the waves go straight on to the next tile of the list;
//   PW waves   stage the operands: global -> NST register stages -> two LDS buffers of 64-deep
//              k-tiles, NST + 1 k-tiles ahead of the multiplication across tile boundaries;
//   CW waves   own the C stream: while tile i is multiplied they combine the staged accumulators of
//              tile i - 1 with that tile's C values (in registers since the pass before) in 16-byte
//              row pieces, store them, and refill each register with the same piece of tile i's C, which
//              then has a whole tile's time to arrive.
// The steps of a tile are unrolled (NK k-tiles per tile, K == 64 NK for every problem of the launch), so
// every wave's instruction stream is static and the waits count exactly the loads that may stay in flight.
// Persistent: workgroup w walks tiles[ranges[w].begin .. ranges[w].end).
constexpr int WS_BK = 64, WS_KP = WS_BK + 8, WS_SP = 132;
constexpr int WS_OP_ELEMS = 2 * 128 * WS_KP;               // bf16 elements of one LDS operand buffer (A tile, B tile)
constexpr int WS_LDS_BYTES = 2 * WS_OP_ELEMS * 2 + 128 * WS_SP * 4;
// cache policy of the C stream: non-temporal (every C value is touched once per launch; with the hint the
// stream takes less of the L2 from the operand panels: 2.73 -> 2.63 ms on the 1B workload, same box, of
// which the stores give all but 0.01)
constexpr int WS_NT = 2;

// PW operand waves with NST register stages, CW waves on the C stream.
template <int NK, int PW, int CW, int NST>
__global__ __launch_bounds__((4 + PW + CW) * 64, 1) void nt_rmw_ws_kernel(const NtLaunch L) {
    static_assert(NK >= 2 && NK % 2 == 0 && NK % NST == 0, "the C waves need NK - 1 steps; stage and buffer of a step are static");
    static_assert((PW == 2 || PW == 4) && (CW == 2 || CW == 4), "row counts below");
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
    float* S = (float*)(lds + 2 * WS_OP_ELEMS);             // staged accumulators, 128 rows of pitch WS_SP

    NtRange range;
    range.begin = nt_const(L.ranges)[blockIdx.x].begin;
    range.end = nt_const(L.ranges)[blockIdx.x].end;
    if (range.begin >= range.end) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ntiles = range.end - range.begin;

    if (wave < 4) {
        // ------------------------------------------------ multiply
        const int wm = wave >> 1, wn = wave & 1;
        f32x16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
        auto compute = [&](int buf) {
            const unsigned short* sA = lds + buf * WS_OP_ELEMS;
            const unsigned short* sB = sA + 128 * WS_KP;
#pragma unroll
            for (int kk = 0; kk < WS_BK / 16; ++kk) {
                const int kofs = kk * 16 + (lane >> 5) * 8;
                bf16x8 fa[2], fb[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) fa[i] = *(const bf16x8*)(sA + (wm * 64 + i * 32 + (lane & 31)) * WS_KP + kofs);
#pragma unroll
                for (int j = 0; j < 2; ++j) fb[j] = *(const bf16x8*)(sB + (wn * 64 + j * 32 + (lane & 31)) * WS_KP + kofs);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        };
        __syncthreads();                                     // k-tile 0 is in LDS buffer 0
        for (int ti = 0; ti < ntiles; ++ti) {
#pragma unroll
            for (int s = 0; s < NK; ++s) {
                compute(s & 1);
                if (s == NK - 1) {
                    // lane holds column (lane & 31); rows 8 (e / 4) + 4 (lane >> 5) + e % 4 of each 32 x 32 tile
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
#pragma unroll
                            for (int e = 0; e < 16; ++e) {
                                const int row = wm * 64 + i * 32 + (lane >> 5) * 4 + (e >> 2) * 8 + (e & 3);
                                S[row * WS_SP + wn * 64 + j * 32 + (lane & 31)] = acc[i][j][e];
                                acc[i][j][e] = 0.0f;
                            }
                }
                __syncthreads();
            }
        }
    } else if (wave < 4 + PW) {
        // ------------------------------------------------ operand stages
        const int ptid = tid - 256;                          // 0 .. 64 PW - 1
        constexpr int CHP = 16 / PW, RSTEP = 8 * PW;         // chunks per thread and operand; rows between them
        int lt = range.begin, lk = 0;                        // loader cursor: tile of the list, k-tile of the tile
        nt_rsrc_t rA, rB;
        unsigned lda_b, ldb_b;
        int row0, col0;
        auto open_tile = [&](int t) {
            const NT_CONST NtTile* tl = nt_const(L.tiles) + t;
            const NT_CONST NtProblem* pp = nt_const(L.probs) + nt_uni(tl->prob);
            const int K = nt_uni(pp->K);
            rA = nt_make_rsrc_uni(pp->A, ((long long)(pp->M - 1) * pp->lda + K) * 2);
            rB = nt_make_rsrc_uni(pp->B, ((long long)(pp->N - 1) * pp->ldb + K) * 2);
            lda_b = (unsigned)nt_uni((int)pp->lda * 2);
            ldb_b = (unsigned)nt_uni((int)pp->ldb * 2);
            row0 = nt_uni(tl->tm * 128); col0 = nt_uni(tl->tn * 128);
        };
        open_tile(lt);
        // chunk c = ptid + 64 PW u of an operand tile: row c / 8, k offset (c % 8) * 8 = (ptid % 8) * 8
        u32x4 sa[NST][CHP], sb[NST][CHP];
        const int crow = ptid >> 3, ck = (ptid & 7) * 8;
        auto load_next = [&](int slot) {                     // unconditional: beyond the list the tile reads as zero
            const unsigned poison = (lt < range.end) ? 0u : 0x80000000u;
            const unsigned kb = (unsigned)(lk * WS_BK + ck) * 2u;
#pragma unroll
            for (int u = 0; u < CHP; ++u) {
                const unsigned va = ((unsigned)(row0 + crow + RSTEP * u) * lda_b + kb) | poison;
                sa[slot][u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rA, (int)va, 0, 0));
            }
#pragma unroll
            for (int u = 0; u < CHP; ++u) {
                const unsigned vb = ((unsigned)(col0 + crow + RSTEP * u) * ldb_b + kb) | poison;
                sb[slot][u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rB, (int)vb, 0, 0));
            }
            if (lt < range.end && ++lk == NK) { lk = 0; if (++lt < range.end) open_tile(lt); }
        };
        auto store = [&](int slot, int buf) {
            unsigned short* d = lds + buf * WS_OP_ELEMS + crow * WS_KP + ck;
#pragma unroll
            for (int u = 0; u < CHP; ++u) *(u32x4*)(d + RSTEP * u * WS_KP) = sa[slot][u];
#pragma unroll
            for (int u = 0; u < CHP; ++u) *(u32x4*)(d + (128 + RSTEP * u) * WS_KP) = sb[slot][u];
        };
        load_next(0);
        store(0, 0);
        __syncthreads();
#pragma unroll
        for (int q = 1; q <= NST; ++q) {                     // k-tiles 1 .. NST into stages 1 .. NST - 1, 0
            load_next(q % NST);
            __builtin_amdgcn_sched_barrier(0);               // keep the issue order: a store waits for the oldest stage only
        }
        // step g: k-tile g is multiplied from buffer g & 1; k-tile g + 1 moves from stage (g + 1) % NST
        // into the other buffer, and that stage is refilled with k-tile g + 1 + NST
        for (int ti = 0; ti < ntiles; ++ti) {
#pragma unroll
            for (int s = 0; s < NK; ++s) {
                store((s + 1) % NST, (s + 1) & 1);
                load_next((s + 1) % NST);
                __syncthreads();
            }
        }
    } else {
        // ------------------------------------------------ C stream
        const int wtid = tid - (4 + PW) * 64;                // 0 .. 64 CW - 1
        constexpr int RP = 2 * CW, NPC = 128 / RP;           // rows per pass of the C waves; pieces per thread
        const int cq = wtid & 31, rb = wtid >> 5;            // piece c of a thread: row rb + RP c, columns 4 cq .. 4 cq + 3
        const float alpha = L.alpha, beta = L.beta;
        // per tile: descriptor and scalars in SGPRs; base = byte offset of this thread's piece 0.  Every piece
        // is one 16-byte load and one 16-byte store whatever the tile (the instruction stream stays static): in
        // a tile on the right edge the piece that would cross column N starts at column N - 4 instead and
        // overlaps its left neighbour, which computes the same values for the shared columns from the same
        // inputs (N % 128 is 0 or at least 4: the host sends nothing else here); pieces wholly beyond N and
        // rows beyond M are dropped through a poisoned offset.
        struct CTile { nt_rsrc_t rc; unsigned base, rowstep; int rows, cs; bool edge; };
        auto open_c = [&](int t, CTile& ct) {
            const bool valid = t < range.end;
            const NT_CONST NtTile* tl = nt_const(L.tiles) + (valid ? t : range.begin);
            const NT_CONST NtProblem* pp = nt_const(L.probs) + nt_uni(tl->prob);
            ct.rc = nt_make_rsrc_uni(pp->C, ((long long)(pp->M - 1) * pp->ldc + pp->N) * 4);
            const unsigned ldc_b = (unsigned)nt_uni((int)pp->ldc * 4);
            const int row0 = nt_uni(tl->tm * 128), col0 = nt_uni(tl->tn * 128);
            const int cols = nt_uni(pp->N) - col0;           // columns of C from the tile's corner on
            ct.edge = cols < 128;
            const int left = cols - 4 * cq;                  // ... and from this thread's piece on
            ct.cs = (left >= 4) ? 4 * cq : cols - 4;
            ct.rows = (valid && left > 0) ? nt_uni(pp->M) - row0 : 0;
            ct.base = (unsigned)(row0 + rb) * ldc_b + (unsigned)(col0 + ct.cs) * 4u;
            ct.rowstep = (unsigned)RP * ldc_b;
        };
        f32x4 wv[NPC];
#pragma unroll
        for (int c = 0; c < NPC; ++c) wv[c] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        CTile prev, cur;
        open_c(range.end, prev);                             // nothing before the first tile: every store is dropped
        open_c(range.begin, cur);
        auto load_piece = [&](const CTile& ct, int c) {
            const unsigned off = (rb + RP * c < ct.rows) ? ct.base + (unsigned)c * ct.rowstep : 0x80000000u;
            wv[c] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(ct.rc, (int)off, 0, WS_NT));
        };
        auto finish_piece = [&](const CTile& ct, int c) {    // staged accumulators + C values of piece c -> memory
            const float* sp = S + (rb + RP * c) * WS_SP;
            f32x4 a;
            if (!ct.edge) {
                a = *(const f32x4*)(sp + 4 * cq);
            } else {                                         // a shifted piece is not 16-byte aligned in LDS
#pragma unroll
                for (int e = 0; e < 4; ++e) a[e] = sp[ct.cs + e];
            }
            f32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (beta == 0.0f) ? alpha * a[e] : alpha * a[e] + beta * wv[c][e];
            const unsigned off = (rb + RP * c < ct.rows) ? ct.base + (unsigned)c * ct.rowstep : 0x80000000u;
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, o), ct.rc, (int)off, 0, WS_NT);
        };
        constexpr int PER = (NPC + NK - 2) / (NK - 1);        // pieces per step, over the first NK - 1 steps of a tile
        __syncthreads();
        for (int ti = 0; ti < ntiles; ++ti) {
#pragma unroll
            for (int s = 0; s < NK; ++s) {
#pragma unroll
                for (int c = s * PER; c < (s + 1) * PER && c < NPC && s < NK - 1; ++c) {
                    finish_piece(prev, c);
                    load_piece(cur, c);
                }
                __syncthreads();
            }
            prev = cur;
            open_c(range.begin + ti + 1, cur);
        }
#pragma unroll
        for (int c = 0; c < NPC; ++c) finish_piece(prev, c); // the last tile of the list
    }
}

// ------------------------------------------------------------------ projection kernel
// RG: groups of 32 rows of V^T (r / 32); wave w owns groups w RG/4 .. and all TN gradient rows.
// DEPTH: k-tiles in flight in registers (gradient tile stages and V^T fragment slots).  A
// workgroup streams its own rows of G from HBM, so the loop runs at memory latency / DEPTH per
// k-tile until DEPTH k-tiles of MFMAs cover that latency.
constexpr int PROJ_BK = 64, PROJ_KP = PROJ_BK + 8;

template <int RG, int TN, int DEPTH>
__device__ __forceinline__ void proj_panel(const ProjItem& it, unsigned short* lds) {
    constexpr int BK = PROJ_BK, KP = PROJ_KP;
    constexpr int FM = RG / 4, FN = TN / 32;
    static_assert(RG % 4 == 0, "r must be a multiple of 128");
    static_assert(DEPTH == 2 || DEPTH == 4, "ring sizes the loop is unrolled for");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int m = it.m, n = it.n, row0 = it.row0;
    const int nsteps = (n + 15) / 16, nk = (n + BK - 1) / BK;
    const nt_rsrc_t rG = nt_make_rsrc(it.G, ((long long)(m - 1) * it.ldg + ((n + 7) & ~7)) * 2);
    const nt_rsrc_t rV = nt_make_rsrc(it.VTf, (long long)RG * nsteps * 1024);
    const unsigned ldg_b = (unsigned)it.ldg * 2u;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    u32x4 af[DEPTH][FM][BK / 16];                            // V^T fragments of DEPTH k-tiles
    auto load_a = [&](int slot, int kt) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                const int s = kt * (BK / 16) + kk;           // steps beyond the last read as zero
                const unsigned voff = (s < nsteps) ? (unsigned)(((wave * FM + i) * nsteps + s) * 64 + lane) * 16u : 0x80000000u;
                af[slot][i][kk] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rV, (int)voff, 0, 0));
            }
    };
    NtStage<TN * BK / 8 / NT_THREADS, false> st[DEPTH];
    auto load_g = [&](int slot, int kt) {
        const int k0 = kt * BK;
        nt_load<TN, BK, false>(st[slot], rG, ldg_b, row0, k0, true, tid);
    };
    const int k_in_tile = (tid % (BK / 8)) * 8;
    auto store_g = [&](int slot, int buf, int kt) {         // kt: the k-tile held by that stage
        const int k0 = kt * BK;
        nt_store<TN, BK, false>(st[slot], lds + buf * (TN * KP), tid, n - (k0 + k_in_tile), k0 + BK > n);
    };
    auto compute = [&](int buf, int slot) {
        const unsigned short* sB = lds + buf * (TN * KP);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int kofs = kk * 16 + h * 8;
            bf16x8 fb[FN];
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = *(const bf16x8*)(sB + (j * 32 + l32) * KP + kofs);
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const bf16x8 fa = __builtin_bit_cast(bf16x8, af[slot][i][kk]);
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb[j], acc[i][j], 0, 0, 0);
            }
        }
    };

    // k-tile kt is multiplied from LDS buffer kt&1 with the fragments in af[kt % DEPTH]; gradient
    // tiles kt+1 .. kt+DEPTH sit in the register stages (tile t in stage t % DEPTH); fragments
    // and stages are refilled in place, DEPTH k-tiles ahead
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (d < nk) { load_g(d, d); load_a(d, d); }
    store_g(0, 0, 0);
    __syncthreads();
    if (DEPTH < nk) load_g(0, DEPTH);
    for (int kt = 0; kt < nk; kt += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const int t = kt + u;                            // uniform; the whole group leaves together
            if (t < nk) {
                compute(u & 1, u);
                if (t + DEPTH < nk) load_a(u, t + DEPTH);
                if (t + 1 < nk) store_g((u + 1) % DEPTH, (u + 1) & 1, t + 1);
                __syncthreads();
                if (t + 1 + DEPTH < nk) load_g((u + 1) % DEPTH, t + 1 + DEPTH);
            }
        }
    }

    // P^T[ri][row]: lane holds gradient row (lane & 31) of each 32-row group, registers run over ri
    const nt_rsrc_t rP = nt_make_rsrc(it.PT, ((long long)(RG * 32 - 1) * it.ldp + m) * 2);
    const unsigned ldp_b = (unsigned)it.ldp * 2u;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int row = row0 + j * 32 + l32;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int ri = (wave * FM + i) * 32 + (e >> 2) * 8 + 4 * h + (e & 3);
                const unsigned vo = (row < m) ? (unsigned)ri * ldp_b + (unsigned)row * 2u : 0x80000000u;
                __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16_bits(acc[i][j][e]), rP, (int)vo, 0, 0);
            }
        }
}

template <int RG, int TN, int DEPTH, int MINB>
__global__ __launch_bounds__(NT_THREADS, MINB) void proj_kernel(const ProjItem* items) {
    __shared__ __attribute__((aligned(16))) unsigned short lds[2 * TN * PROJ_KP];
    const ProjItem it = items[blockIdx.x];
    if (it.G == nullptr) return;
    proj_panel<RG, TN, DEPTH>(it, lds);
}

bool proj_supports_rank(int r) { return r == 128 || r == 256; }

hipError_t launch_proj(const ProjItem* items_dev, int n_items, int r, int depth, hipStream_t stream) {
    if (n_items <= 0) return hipSuccess;
    if (r == 256 && depth == 4) hipLaunchKernelGGL((proj_kernel<8, 128, 4, 1>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else if (r == 256 && depth == 2) hipLaunchKernelGGL((proj_kernel<8, 128, 2, 2>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else if (r == 128) hipLaunchKernelGGL((proj_kernel<4, 128, 4, 2>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------ dispatch
struct NtEntry { int shape, b_f32, out; nt_fn fn; nt_fn persistent; int lds_bytes; int minb; int pieces; };

template <int TM, int TN, int WM, int WN, int BK, bool BF32, int OUT, int MINB>
constexpr nt_fn nt_persistent_fn() {
    if constexpr (OUT == 2) return nullptr;
    else return nt_gemm_persistent_kernel<TM, TN, WM, WN, BK, BF32, OUT, MINB>;
}
// out = 3 (fused Adam) exists as a persistent kernel only, for bf16 operands
#define NT_ENTRY_ADAM(shape, TM, TN, WM, WN, BK, MINB) \
    { shape, 0, 3, nullptr, nt_gemm_persistent_kernel<TM, TN, WM, WN, BK, false, 3, MINB>, 2 * (TM + TN) * (BK + 8) * 2, MINB, 1 }

#define NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, bf32, out) \
    { shape, bf32, out, nt_gemm_kernel<TM, TN, WM, WN, BK, (bf32) != 0, out, MINB>, \
      nt_persistent_fn<TM, TN, WM, WN, BK, (bf32) != 0, out, MINB>(), 2 * (TM + TN) * (BK + 8) * 2, MINB, 1 }
// fp32 output, B in NP bf16 pieces
#define NT_ENTRY_PIECES(shape, TM, TN, WM, WN, BK, MINB, NP) \
    { shape, 0, 0, nt_gemm_kernel<TM, TN, WM, WN, BK, false, 0, MINB, NP>, nullptr, 2 * (TM + (NP) * TN) * (BK + 8) * 2, MINB, NP }
// MINB / MINB_RMW: workgroups per CU the register allocation must allow (the read-modify-write
// variant also holds the C tile in registers)
#define NT_SHAPE(shape, TM, TN, WM, WN, BK, MINB, MINB_RMW)                                                   \
    NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 0, 0), NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 0, 1),         \
    NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB_RMW, 0, 2), NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 1, 0),     \
    NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 1, 1)

static const NtEntry kNt[] = {
    NT_SHAPE(NT_128x128, 128, 128, 2, 2, 64, 2, 1), NT_SHAPE(NT_64x256, 64, 256, 1, 4, 64, 1, 1),
    NT_SHAPE(NT_64x64, 64, 64, 2, 2, 64, 4, 4),
    NT_ENTRY_ADAM(NT_64x64, 64, 64, 2, 2, 64, 4),
    { NT_256x256_K32, 0, 0, nt_wide_kernel<4, 4, 1, 0>, nullptr, 2 * (256 + 256) * 32 * 2, 1, 1 },
    { NT_256x256_K32, 0, 1, nt_wide_kernel<4, 4, 1, 1>, nullptr, 2 * (256 + 256) * 32 * 2, 1, 1 },
    { NT_256x128_K32, 0, 0, nt_wide_kernel<4, 2, 2, 0>, nullptr, 2 * (256 + 2 * 128) * 32 * 2, 1, 2 },
    NT_ENTRY_PIECES(NT_128x128_K32, 128, 128, 2, 2, 32, 2, 2),
};

hipError_t launch_nt_gemm(const NtLaunch& L, const NtVariant& v, hipStream_t stream) {
    if (L.n_tiles <= 0) return hipSuccess;
    if (v.shape == NT_128x128_WS) {
        if (!L.ranges || v.b_f32 || v.out_bf16 || v.fused_adam || v.b_pieces > 1) return hipErrorInvalidValue;
        const nt_fn fn = nt_rmw_ws_kernel<8, 4, 4, 4>;
        constexpr int threads = (4 + 4 + 4) * 64;
        static thread_local bool configured_ws = false;
        if (!configured_ws) {
            hipError_t er = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, WS_LDS_BYTES);
            if (er != hipSuccess) return er;
            configured_ws = true;
        }
        hipLaunchKernelGGL(fn, dim3(L.n_tiles), dim3(threads), WS_LDS_BYTES, stream, L);
        return hipGetLastError();
    }
    const int out = v.fused_adam ? 3 : (v.out_bf16 ? 1 : (L.beta != 0.0f ? 2 : 0));
    for (const NtEntry& e : kNt) {
        if (e.shape == v.shape && e.b_f32 == v.b_f32 && e.out == out && e.pieces == (v.b_pieces > 1 ? v.b_pieces : 1)) {
            const nt_fn fn = L.ranges ? e.persistent : e.fn;
            if (fn == nullptr) return hipErrorInvalidValue;
            static thread_local const void* configured[256] = {nullptr};
            bool done = false;
            for (const void* c : configured) if (c == (const void*)fn) { done = true; break; }
            if (!done) {
                hipError_t er = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                    e.lds_bytes);
                if (er != hipSuccess) return er;
                for (const void*& c : configured) if (c == nullptr) { c = (const void*)fn; break; }
            }
            hipLaunchKernelGGL(fn, dim3(L.n_tiles), dim3(NT_THREADS), e.lds_bytes, stream, L);
            return hipGetLastError();
        }
    }
    return hipErrorInvalidValue;
}

int nt_wgs_per_cu(int shape) {
    for (const NtEntry& e : kNt) if (e.shape == shape && e.out == 0 && e.pieces == 1) return e.minb;
    return 1;
}

// ------------------------------------------------------------------ bf16 shadows of the bases
// One workgroup converts a 64 x 64 patch: Xb[row][c] and, through LDS, XTb[c][row].
__global__ __launch_bounds__(256) void shadow_kernel(const ShadowBlock* table) {
    const ShadowBlock b = table[blockIdx.z];
    const int rows = b.rows, r = b.r;
    const int row0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    // patches cover the padded extents (ldx columns, ldt columns of the transpose)
    if (row0 >= (int)b.ldt || c0 >= (int)b.ldx) return;
    __shared__ unsigned short tile[64][66];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    unsigned short* Xb = (unsigned short*)b.Xb;
    unsigned short* XTb = (unsigned short*)b.XTb;
    unsigned short* XFb = (unsigned short*)b.XFb;
    unsigned short* XTFb = (unsigned short*)b.XTFb;
    const int rows32 = (rows + 31) / 32 * 32, ksteps = r / 16;
    const int rows16 = (rows + 15) / 16 * 16, nsteps = rows16 / 16;
    for (int i = ty; i < 64; i += 4) {
        const int row = row0 + i, c = c0 + tx;
        const float v = (row < rows && c < r) ? b.X[(long long)row * r + c] : 0.0f;
        const unsigned short h = f32_to_bf16_bits(v);
        tile[i][tx] = h;
        if (row < rows && c < (int)b.ldx) Xb[(long long)row * b.ldx + c] = h;
        if (XFb && row < rows32 && c < r)
            XFb[(((long long)(row / 32) * ksteps + c / 16) * 64 + ((c % 16) / 8) * 32 + row % 32) * 8 + c % 8] = h;
        if (XTFb && row < rows16 && c < r)
            XTFb[(((long long)(c / 32) * nsteps + row / 16) * 64 + ((row % 16) / 8) * 32 + c % 32) * 8 + row % 8] = h;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int c = c0 + i, row = row0 + tx;
        if (c < r && row < (int)b.ldt) XTb[(long long)c * b.ldt + row] = tile[tx][i];
    }
}

hipError_t launch_shadows(const ShadowBlock* table_dev, int blocks, int max_rows, int max_r, hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    dim3 grid((max_r + 8 + 63) / 64, (max_rows + 8 + 63) / 64, blocks);
    hipLaunchKernelGGL(shadow_kernel, grid, dim3(256), 0, stream, table_dev);
    return hipGetLastError();
}

// ------------------------------------------------------------------ operands of the refresh GEMMs
// 64 x 64 patches through LDS; element pairs (4 bytes) on both sides.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const TransposeBlock* table) {
    const TransposeBlock b = table[blockIdx.z];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    if (r0 >= (int)b.ld_dst || c0 >= b.cols) return;
    __shared__ unsigned short tile[64][66];
    const unsigned short* src = (const unsigned short*)b.src;
    unsigned short* dst = (unsigned short*)b.dst;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;          // 32 pairs across, 8 rows per pass
    for (int i = ty; i < 64; i += 8) {
        const int r = r0 + i, c = c0 + 2 * tx;
        unsigned v = 0u;
        if (r < b.rows) {
            if (c + 1 < b.cols) v = *(const unsigned*)(src + (long long)r * b.ld_src + c);
            else if (c < b.cols) v = src[(long long)r * b.ld_src + c];
        }
        tile[i][2 * tx] = (unsigned short)(v & 0xffffu);
        tile[i][2 * tx + 1] = (unsigned short)(v >> 16);
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 8) {
        const int c = c0 + i, r = r0 + 2 * tx;                       // dst[c][r], dst[c][r + 1]
        if (c < b.cols && r < (int)b.ld_dst)
            *(unsigned*)(dst + (long long)c * b.ld_dst + r) = (unsigned)tile[2 * tx][i] | ((unsigned)tile[2 * tx + 1][i] << 16);
    }
}

hipError_t launch_transpose_bf16(const TransposeBlock* table_dev, int blocks, int max_rows, int max_cols, hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    dim3 grid((max_cols + 63) / 64, (max_rows + 8 + 63) / 64, blocks);
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, stream, table_dev);
    return hipGetLastError();
}

template <int PIECES>
__global__ __launch_bounds__(256) void split_transpose_kernel(const SplitBlock* table) {
    const SplitBlock b = table[blockIdx.z];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int rows8 = (b.rows + 7) / 8 * 8;                         // written width of an output row (zeros beyond `rows`)
    if (r0 >= rows8 || c0 >= b.k) return;
    __shared__ unsigned short tile[PIECES][64][66];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        float x = (r < b.rows && c < b.k) ? b.X[(long long)r * b.k + c] : 0.0f;
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const __bf16 h = (__bf16)x;
            tile[p][i][tx] = __builtin_bit_cast(unsigned short, h);
            x -= (float)h;
        }
    }
    __syncthreads();
    unsigned short* dst = (unsigned short*)b.dst;
    const int px = threadIdx.x & 31, py = threadIdx.x >> 5;
    for (int i = py; i < 64; i += 8) {
        const int c = c0 + i, r = r0 + 2 * px;                       // piece[c][r], piece[c][r + 1]
        if (c < b.k && r < rows8) {
#pragma unroll
            for (int p = 0; p < PIECES; ++p)
                *(unsigned*)(dst + (long long)p * b.piece_stride + (long long)c * b.ld_dst + r) =
                    (unsigned)tile[p][2 * px][i] | ((unsigned)tile[p][2 * px + 1][i] << 16);
        }
    }
}

hipError_t launch_split_transpose(const SplitBlock* table_dev, int blocks, int max_rows, int max_k, int pieces,
                                  hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    dim3 grid((max_k + 63) / 64, (max_rows + 8 + 63) / 64, blocks);
    if (pieces == 2) hipLaunchKernelGGL(split_transpose_kernel<2>, grid, dim3(256), 0, stream, table_dev);
    else if (pieces == 3) hipLaunchKernelGGL(split_transpose_kernel<3>, grid, dim3(256), 0, stream, table_dev);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

template <int PIECES>
__global__ __launch_bounds__(256) void split_rows_kernel(const SplitBlock* table) {
    const SplitBlock b = table[blockIdx.z];
    const int wp = (b.k + 7) / 8 * 4;                                   // element pairs written per output row (zeros beyond k)
    const long long pairs = (long long)b.rows * wp;
    unsigned* dst = (unsigned*)b.dst;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < pairs; i += (long long)gridDim.x * 256) {
        const int r = (int)(i / wp), c = (int)(i % wp) * 2;
        float x0 = (c < b.k) ? b.X[(long long)r * b.k + c] : 0.0f;
        float x1 = (c + 1 < b.k) ? b.X[(long long)r * b.k + c + 1] : 0.0f;
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const __bf16 h0 = (__bf16)x0, h1 = (__bf16)x1;
            dst[((long long)p * b.piece_stride + (long long)r * b.ld_dst + c) / 2] =
                (unsigned)__builtin_bit_cast(unsigned short, h0) | ((unsigned)__builtin_bit_cast(unsigned short, h1) << 16);
            x0 -= (float)h0; x1 -= (float)h1;
        }
    }
}

hipError_t launch_split_rows(const SplitBlock* table_dev, int blocks, int max_rows, int max_k, int pieces, hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    long long bx = ((long long)max_rows * ((max_k + 8) / 2) + 255) / 256;
    if (bx > 2048) bx = 2048;
    dim3 grid((unsigned)bx, 1, blocks);
    if (pieces == 2) hipLaunchKernelGGL(split_rows_kernel<2>, grid, dim3(256), 0, stream, table_dev);
    else if (pieces == 3) hipLaunchKernelGGL(split_rows_kernel<3>, grid, dim3(256), 0, stream, table_dev);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace tsr
