// bf16 NT GEMM for the per-step path on gfx950: C = alpha A B^T + beta C with A (M x K) and
// B (N x K) both k-contiguous.  256 threads, 64-deep k-tiles, double-buffered LDS (one
// barrier per k-tile), register prefetch of the next k-tile, v_mfma_f32_32x32x16_bf16 with
// fp32 accumulation.  For the read-modify-write epilogue (beta != 0) the C tile is fetched
// before the k-loop so that its HBM latency hides behind the whole loop.
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

// rows x K operand, k contiguous; tile rows row0.., k0..k0+BK-1.  Thread t owns chunks
// c = t + 256*it: row c/(BK/8), k offset (c%(BK/8))*8.  `tail`: this k-tile crosses kend.
template <int ROWS, int BK, bool F32>
__device__ inline void nt_load(NtStage<ROWS * BK / 8 / NT_THREADS, F32>& s, nt_rsrc_t rs, unsigned ld_bytes, int row0,
                               int k0, int kend, bool tail, int tid) {
    constexpr int CPR = BK / 8;
    constexpr int ESZ = F32 ? 4 : 2;
    constexpr int CH = ROWS * CPR / NT_THREADS;
#pragma unroll
    for (int it = 0; it < CH; ++it) {
        const int c = tid + NT_THREADS * it;
        const unsigned grow = row0 + c / CPR;
        const int gk = k0 + (c % CPR) * 8;
        const unsigned voff = grow * ld_bytes + (unsigned)gk * ESZ;
        if constexpr (F32) {
            s.v[it][0] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, 0, 0));
            s.v[it][1] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(voff + 16), 0, 0));
        } else {
            s.v[it] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, 0, 0));
        }
    }
    if (tail) {                                             // wave-uniform: last k-tile only
#pragma unroll
        for (int it = 0; it < CH; ++it) {
            const int c = tid + NT_THREADS * it;
            const int valid = kend - (k0 + (c % CPR) * 8);  // elements of this chunk inside [.., kend)
            if constexpr (F32) {
                u32x4 m0, m1;
#pragma unroll
                for (int j = 0; j < 4; ++j) { m0[j] = (j < valid) ? 0xffffffffu : 0u; m1[j] = (4 + j < valid) ? 0xffffffffu : 0u; }
                s.v[it][0] = __builtin_bit_cast(f32x4, __builtin_bit_cast(u32x4, s.v[it][0]) & m0);
                s.v[it][1] = __builtin_bit_cast(f32x4, __builtin_bit_cast(u32x4, s.v[it][1]) & m1);
            } else {
                u32x4 m;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    m[j] = ((2 * j < valid) ? 0x0000ffffu : 0u) | ((2 * j + 1 < valid) ? 0xffff0000u : 0u);
                s.v[it] = s.v[it] & m;
            }
        }
    }
}

template <int ROWS, int BK, bool F32>
__device__ inline void nt_store(const NtStage<ROWS * BK / 8 / NT_THREADS, F32>& s, unsigned short* lds, int tid) {
    constexpr int CPR = BK / 8, KP = BK + 8;
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
}

__device__ inline unsigned short f32_to_bf16_bits(float f) {
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(unsigned short, h);
}

// OUT: 0 = fp32 store (alpha only), 1 = bf16 store (alpha only), 2 = fp32 read-modify-write
template <int TM, int TN, int WM, int WN, int NT_BK, bool B_F32, int OUT, int MINB>
__global__ __launch_bounds__(NT_THREADS, MINB) void nt_gemm_kernel(const NtLaunch L) {
    constexpr bool OUT_BF16 = (OUT == 1);
    constexpr bool RMW = (OUT == 2);
    static_assert(WM * WN == 4, "four waves");
    constexpr int NT_KP = NT_BK + 8;
    constexpr int FM = TM / WM / 32, FN = TN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned short lds[];
    constexpr int A_ELEMS = TM * NT_KP, B_ELEMS = TN * NT_KP, BUF = A_ELEMS + B_ELEMS;

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
    const nt_rsrc_t rB = nt_make_rsrc(B, ((long long)(N - 1) * ldb + k8) * (B_F32 ? 4 : 2));
    const unsigned lda_b = (unsigned)lda * 2u, ldb_b = (unsigned)ldb * (B_F32 ? 4u : 2u);

    // For the read-modify-write epilogue the C tile is fetched into registers before the k-loop
    // and only consumed after it, so its HBM latency hides behind the whole loop.
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
    if constexpr (RMW) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    cold[i][j][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rC, (int)c_voff(i, j, e), 0, 0));
    }
    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Two k-tiles travel in registers ahead of the one being multiplied (ring of two register
    // stages), one more sits in the other LDS buffer: global latency hides behind two k-tiles of
    // MFMAs per workgroup.  The read-modify-write variant keeps one stage only (its k-loop is
    // short and its registers hold the C tile).
    constexpr int NSTAGE = RMW ? 1 : 2;
    NtStage<TM * NT_BK / 8 / NT_THREADS, false> stA[NSTAGE];
    NtStage<TN * NT_BK / 8 / NT_THREADS, B_F32> stB[NSTAGE];
    const int nk = (kend > kbeg && !skip_products) ? (kend - kbeg + NT_BK - 1) / NT_BK : 0;

    auto load = [&](int slot, int tile) {
        const int k0 = kbeg + tile * NT_BK;
        const bool tail = k0 + NT_BK > kend;
        nt_load<TM, NT_BK, false>(stA[slot], rA, lda_b, row0, k0, kend, tail, tid);
        nt_load<TN, NT_BK, B_F32>(stB[slot], rB, ldb_b, col0, k0, kend, tail, tid);
    };
    auto store = [&](int slot, int buf) {
        unsigned short* d = lds + buf * BUF;
        nt_store<TM, NT_BK, false>(stA[slot], d, tid);
        nt_store<TN, NT_BK, B_F32>(stB[slot], d + A_ELEMS, tid);
    };
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

    if constexpr (NSTAGE == 2) {
        // prologue: tile 0 -> LDS buffer 0; tiles 1 and 2 -> register stages 1 and 0
        if (nk > 0) {
            load(0, 0);
            store(0, 0);
            __syncthreads();
            if (nk > 1) load(1, 1);
            if (nk > 2) load(0, 2);
        }
        // iteration `it` multiplies LDS buffer it&1, moves tile it+1 (register stage (it+1)&1) into
        // the other buffer and refills that stage with tile it+3
        for (int it = 0; it < nk; it += 2) {
            compute(0);
            if (it + 1 < nk) store(1, 1);
            __syncthreads();
            if (it + 3 < nk) load(1, it + 3);
            if (it + 1 < nk) {
                compute(1);
                if (it + 2 < nk) store(0, 0);
                __syncthreads();
                if (it + 4 < nk) load(0, it + 4);
            }
        }
    } else {
        if (nk > 0) {
            load(0, 0);
            store(0, 0);
            __syncthreads();
            if (nk > 1) load(0, 1);
        }
        for (int it = 0; it < nk; ++it) {
            compute(it & 1);
            if (it + 1 < nk) store(0, (it + 1) & 1);
            __syncthreads();
            if (it + 2 < nk) load(0, it + 2);
        }
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
    auto load_next = [&](int slot) {
        const int k0 = l_kbeg + lk * NT_BK;
        const bool tail = k0 + NT_BK > l_kend;
        nt_load<TM, NT_BK, false>(stA[slot], rA, lda_b, l_row0, k0, l_kend, tail, tid);
        nt_load<TN, NT_BK, B_F32>(stB[slot], rB, ldb_b, l_col0, k0, l_kend, tail, tid);
        if (++lk == l_nk) { lk = 0; if (++lt < range.end) open_tile(lt); }
    };
    auto store = [&](int slot, int buf) {
        unsigned short* d = lds + buf * BUF;
        nt_store<TM, NT_BK, false>(stA[slot], d, tid);
        nt_store<TN, NT_BK, B_F32>(stB[slot], d + A_ELEMS, tid);
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
    if (total > 1) load_next(1);
    if (total > 2) load_next(0);
    for (int g = 0; g < total; g += 2) {
        compute(0);
        finish_step();
        if (g + 1 < total) store(1, 1);
        __syncthreads();
        if (g + 3 < total) load_next(1);
        if (g + 1 < total) {
            compute(1);
            finish_step();
            if (g + 2 < total) store(0, 0);
            __syncthreads();
            if (g + 4 < total) load_next(0);
        }
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
        nt_load<TN, BK, false>(st[slot], rG, ldg_b, row0, k0, n, k0 + BK > n, tid);
    };
    auto store_g = [&](int slot, int buf) { nt_store<TN, BK, false>(st[slot], lds + buf * (TN * KP), tid); };
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
    store_g(0, 0);
    __syncthreads();
    if (DEPTH < nk) load_g(0, DEPTH);
    for (int kt = 0; kt < nk; kt += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const int t = kt + u;                            // uniform; the whole group leaves together
            if (t < nk) {
                compute(u & 1, u);
                if (t + DEPTH < nk) load_a(u, t + DEPTH);
                if (t + 1 < nk) store_g((u + 1) % DEPTH, (u + 1) & 1);
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

hipError_t launch_proj(const ProjItem* items_dev, int n_items, int r, int panel_rows, hipStream_t stream) {
    if (n_items <= 0) return hipSuccess;
    if (r == 256 && panel_rows == 128) hipLaunchKernelGGL((proj_kernel<8, 128, 4, 1>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else if (r == 256 && panel_rows == 129) hipLaunchKernelGGL((proj_kernel<8, 128, 2, 2>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else if (r == 256 && panel_rows == 64) hipLaunchKernelGGL((proj_kernel<8, 64, 4, 2>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else if (r == 128 && panel_rows >= 128) hipLaunchKernelGGL((proj_kernel<4, 128, 4, 2>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else if (r == 128 && panel_rows == 64) hipLaunchKernelGGL((proj_kernel<4, 64, 4, 3>), dim3(n_items), dim3(NT_THREADS), 0, stream, items_dev);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------ dispatch
typedef void (*nt_fn)(const NtLaunch);
struct NtEntry { int shape, b_f32, out; nt_fn fn; nt_fn persistent; int lds_bytes; int minb; };

template <int TM, int TN, int WM, int WN, int BK, bool BF32, int OUT, int MINB>
constexpr nt_fn nt_persistent_fn() {
    if constexpr (OUT == 2) return nullptr;
    else return nt_gemm_persistent_kernel<TM, TN, WM, WN, BK, BF32, OUT, MINB>;
}
// out = 3 (fused Adam) exists as a persistent kernel only, for bf16 operands
#define NT_ENTRY_ADAM(shape, TM, TN, WM, WN, BK, MINB) \
    { shape, 0, 3, nullptr, nt_gemm_persistent_kernel<TM, TN, WM, WN, BK, false, 3, MINB>, 2 * (TM + TN) * (BK + 8) * 2, MINB }

#define NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, bf32, out) \
    { shape, bf32, out, nt_gemm_kernel<TM, TN, WM, WN, BK, (bf32) != 0, out, MINB>, \
      nt_persistent_fn<TM, TN, WM, WN, BK, (bf32) != 0, out, MINB>(), 2 * (TM + TN) * (BK + 8) * 2, MINB }
// MINB / MINB_RMW: workgroups per CU the register allocation must allow (the read-modify-write
// variant also holds the C tile in registers)
#define NT_SHAPE(shape, TM, TN, WM, WN, BK, MINB, MINB_RMW)                                                   \
    NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 0, 0), NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 0, 1),         \
    NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB_RMW, 0, 2), NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 1, 0),     \
    NT_ENTRY(shape, TM, TN, WM, WN, BK, MINB, 1, 1)

static const NtEntry kNt[] = {
    NT_SHAPE(NT_128x128, 128, 128, 2, 2, 64, 2, 1), NT_SHAPE(NT_256x64, 256, 64, 4, 1, 64, 1, 1),
    NT_SHAPE(NT_64x256, 64, 256, 1, 4, 64, 1, 1),   NT_SHAPE(NT_64x64, 64, 64, 2, 2, 64, 4, 4),
    NT_SHAPE(NT_128x128_K32, 128, 128, 2, 2, 32, 3, 2), NT_SHAPE(NT_256x64_K32, 256, 64, 4, 1, 32, 3, 2),
    NT_SHAPE(NT_256x128_K32, 256, 128, 2, 2, 32, 2, 1), NT_SHAPE(NT_128x256_K32, 128, 256, 2, 2, 32, 2, 1),
    NT_SHAPE(NT_256x128, 256, 128, 2, 2, 64, 1, 1),
    NT_ENTRY_ADAM(NT_64x64, 64, 64, 2, 2, 64, 4),
};

hipError_t launch_nt_gemm(const NtLaunch& L, const NtVariant& v, hipStream_t stream) {
    if (L.n_tiles <= 0) return hipSuccess;
    const int out = v.fused_adam ? 3 : (v.out_bf16 ? 1 : (L.beta != 0.0f ? 2 : 0));
    for (const NtEntry& e : kNt) {
        if (e.shape == v.shape && e.b_f32 == v.b_f32 && e.out == out) {
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
    for (const NtEntry& e : kNt) if (e.shape == shape && e.out == 0) return e.minb;
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

}  // namespace tsr
