// Fused back-projection + weight update for the bf16 step path on gfx950:
//     W <- beta W + alpha (U D) V^T           (alpha = -lr*scale, beta = 1 - lr*wd)
// The launch is persistent: each workgroup (4 waves) walks its own list of work items, an item
// being a 128-row panel of one block and a run of 128-column tiles; the host cuts the tiles of
// all blocks into equally heavy lists, one per workgroup.  Per item:
//   setup : T = alpha U_panel D (128 x r) is computed once with MFMAs (U panel staged in LDS,
//           D^T fragments straight from L2) and parked in LDS as bf16;
//   stream: each wave owns 32 of the tile's 128 columns.  Its V fragments (32 columns x r)
//           come straight from global memory in MFMA operand layout and its W values are
//           loaded in accumulator layout, one tile ahead, so nothing but T touches LDS and the
//           streaming loop has no barriers.  W crosses HBM exactly once each way and neither T
//           nor U D V^T is ever written to memory.
// V and D^T are read from copies stored in fragment order (one contiguous 1 KiB record per
// wave-level load, written by the shadow and Adam kernels).  The default variant works on
// 256-row items (two T panels in LDS, one workgroup per CU): V is re-read once per item, and
// these re-reads rarely hit in L2 (the W stream has pushed them out), so taller items are what
// cuts the traffic beyond W itself.
#include "lift.h"

namespace tsr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int LIFT_THREADS = 256;
constexpr int LIFT_TM = 128;                   // rows of a panel

// Raw buffer access: one SGPR descriptor per array, a 32-bit per-lane byte offset plus a
// wave-uniform byte offset.  The hardware range check covers the per-lane offset only (not
// the wave-uniform one): a per-lane offset at or beyond the descriptor's size reads as zero and
// drops the store.  Guards therefore poison the per-lane offset with OOB_LANE.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr int BUF_FLAGS = 0x00020000;          // gfx9 raw buffer, 32-bit data format
constexpr unsigned OOB_LANE = 0x80000000u;
__device__ inline rsrc_t make_rsrc(const void* p, long long bytes) {
    const int n = (bytes > 0x7fffffffLL) ? 0x7fffffff : (int)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), (short)0, n, BUF_FLAGS);
}
__device__ inline u32x4 buf_load128(rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0));
}
// W is touched once per step: its loads and stores carry the non-temporal hint (aux bit 1) so that
// the stream does not push the reused operands (V, D^T, U) out of L2.
#ifndef LIFT_W_AUX
#define LIFT_W_AUX 2
#endif
__device__ inline float buf_load32(rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, LIFT_W_AUX));
}
__device__ inline void buf_store32(float v, rsrc_t r, unsigned voff, unsigned soff) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)voff, (int)soff, LIFT_W_AUX);
}

// PIPE: 1 = prefetch the next tile's V fragments and W values while the current tile is
// multiplied (one workgroup per CU); 2 = W one tile ahead, V fragments reloaded in place as soon
// as the MFMAs of their k step are issued (fewer registers: two workgroups per CU).
// HALVES: 128-row panels per item (1 or 2).  With 2 the item is a 256-row panel: both T halves
// sit in LDS and every V fragment, once in registers, serves both, which halves the V traffic.
template <int KSTEPS, int PIPE, int HALVES, int MINB>
__global__ __launch_bounds__(LIFT_THREADS, MINB) void lift_kernel(const LiftBlock* blocks, const LiftTile* tiles,
                                                                  const LiftRange* ranges, const float alpha,
                                                                  const float beta) {
    constexpr int R = KSTEPS * 16;
    constexpr int XP = R + 8;                 // padded LDS row (bf16 elements)
    constexpr int RT = LIFT_TM / 32;          // 32-row tiles of the panel
    constexpr int CPR = R / 8;                // 16-byte chunks per row of U
    constexpr int PER_THREAD = LIFT_TM * CPR / LIFT_THREADS;
    constexpr int NCT = R / 32;               // 32-wide column tiles of T
    constexpr int CT_W = (NCT >= 4) ? NCT / 4 : 1;            // T column tiles per wave (setup)
    constexpr int WAVES_PER_CT = (NCT >= 4) ? 1 : 4 / NCT;
    constexpr int RT_W = RT / WAVES_PER_CT;                   // T row tiles per wave (setup)
    extern __shared__ __attribute__((aligned(16))) unsigned short X[];   // [HALVES][LIFT_TM][XP]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const LiftRange range = ranges[blockIdx.x];
    const bool skip = (alpha == 0.0f);          // zero learning rate: no products at all

    struct VFrag { u32x4 v[KSTEPS]; };
    struct Acc { f32x16 a[RT]; };
    for (int item = range.begin; item < range.end; ++item) {
        const LiftTile t = tiles[item];
        const LiftBlock b = blocks[t.block];
        const int row0 = t.row0;
        const int ct0 = t.ct0, nct = t.nct;

        const rsrc_t rU = make_rsrc(b.Ub, (long long)b.m * b.ldr * 2);
        const rsrc_t rD = make_rsrc(b.DTf, (long long)b.r * b.r * 2);
        const rsrc_t rV = make_rsrc(b.Vf, (long long)((b.n + 31) / 32) * KSTEPS * 1024);
        const rsrc_t rW = make_rsrc(b.W, ((long long)(b.m - 1) * b.ldw + b.n) * 4);
        const unsigned ldr_b = (unsigned)b.ldr * 2u, ldw_b = (unsigned)b.ldw * 4u;

        // ---- stream helpers: W tile columns ct*128 + wave*32 + l32
        // The W tile is loaded (one tile ahead) straight into the accumulator registers of the
        // tile it belongs to and scaled by beta there; T carries the factor alpha, so the MFMAs
        // leave the updated tile.  A tile that lies wholly inside the matrix (wave-uniform test)
        // needs no guards; elsewhere every access poisons the per-lane offset of elements outside.
        unsigned row_soff[16];                  // byte offset of accumulator row e within a 32-row tile
#pragma unroll
        for (int e = 0; e < 16; ++e) row_soff[e] = (unsigned)((e >> 2) * 8 + (e & 3)) * ldw_b;
        constexpr int halves = HALVES;          // a lower half beyond the matrix is all guards: zero T, nothing stored
        auto v_voff = [&](int ct) -> unsigned {
            // one contiguous 1 KiB record per k step; column groups beyond n read as zero
            return (unsigned)((ct * 4 + wave) * KSTEPS * 64 + lane) * 16u;
        };
        auto load_v = [&](VFrag& f, int ct) {
            const unsigned voff = v_voff(ct);
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) f.v[s] = buf_load128(rV, voff + s * 1024, 0);
        };
        auto w_voff = [&](int ct, int half) -> unsigned {   // element (first row + 4 h, col) of the tile
            return (unsigned)(row0 + half * LIFT_TM + h * 4) * ldw_b + (unsigned)(ct * 128 + wave * 32 + l32) * 4u;
        };
        auto load_w = [&](Acc& w, int ct, int half) {
            const unsigned voff = w_voff(ct, half);
            const int r0 = row0 + half * LIFT_TM;
            if (r0 + LIFT_TM <= b.m && (ct + 1) * 128 <= b.n) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const unsigned vo = voff + (unsigned)(rt * 32) * ldw_b;
#pragma unroll
                    for (int e = 0; e < 16; ++e) w.a[rt][e] = buf_load32(rW, vo, row_soff[e]);
                }
            } else {
                const bool col_ok = ct * 128 + wave * 32 + l32 < b.n;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int dr = rt * 32 + (e >> 2) * 8 + (e & 3);
                        const bool ok = col_ok && (r0 + h * 4 + dr < b.m);
                        w.a[rt][e] = buf_load32(rW, ok ? voff + (unsigned)(rt * 32) * ldw_b : OOB_LANE, row_soff[e]);
                    }
            }
        };
        // next_ct >= 0 (PIPE == 2): reload each k step's V fragment for that tile once it is used
        auto compute_store = [&](VFrag& f, Acc& w, int ct, int half, int next_ct) {
            const unsigned short* Xh = X + half * (LIFT_TM * XP);
            const int r0 = row0 + half * LIFT_TM;
            if (beta != 1.0f) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) w.a[rt][e] *= beta;
            }
            if (!skip) {
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    const int kofs = s * 16 + h * 8;               // the k order of the V records
                    const bf16x8 fv = __builtin_bit_cast(bf16x8, f.v[s]);
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        const bf16x8 ft = *(const bf16x8*)(Xh + (rt * 32 + l32) * XP + kofs);
                        w.a[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ft, fv, w.a[rt], 0, 0, 0);
                    }
                    if constexpr (PIPE == 2) {
                        if (next_ct >= 0) f.v[s] = buf_load128(rV, v_voff(next_ct) + s * 1024, 0);
                    }
                }
            }
            const unsigned voff = w_voff(ct, half);
            if (r0 + LIFT_TM <= b.m && (ct + 1) * 128 <= b.n) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const unsigned vo = voff + (unsigned)(rt * 32) * ldw_b;
#pragma unroll
                    for (int e = 0; e < 16; ++e) buf_store32(w.a[rt][e], rW, vo, row_soff[e]);
                }
            } else {
                const bool col_ok = ct * 128 + wave * 32 + l32 < b.n;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int dr = rt * 32 + (e >> 2) * 8 + (e & 3);
                        const bool ok = col_ok && (r0 + h * 4 + dr < b.m);
                        buf_store32(w.a[rt][e], rW, ok ? voff + (unsigned)(rt * 32) * ldw_b : OOB_LANE, row_soff[e]);
                    }
            }
        };
        VFrag va;
        Acc wa;
        if (item != range.begin) __syncthreads();             // the previous item's T panel is no longer read

#pragma unroll
        for (int half = 0; half < halves; ++half) {
        unsigned short* Xh = X + half * (LIFT_TM * XP);
        const int r0 = row0 + half * LIFT_TM;
        // ---- setup 1: U panel -> LDS (rows beyond m read as zero)
        {
            constexpr int GRP = PER_THREAD < 8 ? PER_THREAD : 8;
#pragma unroll
            for (int g = 0; g < PER_THREAD; g += GRP) {
                u32x4 v[GRP];
#pragma unroll
                for (int u = 0; u < GRP; ++u) {
                    const int c = tid + LIFT_THREADS * (g + u);
                    v[u] = buf_load128(rU, (unsigned)(r0 + c / CPR) * ldr_b + (c % CPR) * 16, 0);
                }
#pragma unroll
                for (int u = 0; u < GRP; ++u) {
                    const int c = tid + LIFT_THREADS * (g + u);
                    *(u32x4*)(Xh + (c / CPR) * XP + (c % CPR) * 8) = v[u];
                }
            }
        }
        __syncthreads();

        // ---- setup 2: T^T tiles = D^T (rows c) x U_panel^T (columns row): acc[ct][rt]
        {
            const int ct_base = (NCT >= 4) ? wave * CT_W : wave % NCT;
            const int rt_base = (NCT >= 4) ? 0 : (wave / NCT) * RT_W;
            f32x16 acc[CT_W][RT_W];
#pragma unroll
            for (int i = 0; i < CT_W; ++i)
#pragma unroll
                for (int j = 0; j < RT_W; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
#pragma unroll 4
            for (int s = 0; s < KSTEPS; ++s) {
                const int kofs = s * 16 + h * 8;
                bf16x8 fd[CT_W], fu[RT_W];
#pragma unroll
                for (int i = 0; i < CT_W; ++i)
                    fd[i] = __builtin_bit_cast(bf16x8, buf_load128(rD, (unsigned)(((ct_base + i) * KSTEPS + s) * 64 + lane) * 16u, 0));
#pragma unroll
                for (int j = 0; j < RT_W; ++j) fu[j] = *(const bf16x8*)(Xh + ((rt_base + j) * 32 + l32) * XP + kofs);
#pragma unroll
                for (int i = 0; i < CT_W; ++i)
#pragma unroll
                    for (int j = 0; j < RT_W; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[i], fu[j], acc[i][j], 0, 0, 0);
            }
            __syncthreads();                                  // every wave is done reading U from X
            // acc element e of tile (ct, rt): T column c = ct*32 + 8*(e/4) + 4*h + e%4, T row = rt*32 + l32
#pragma unroll
            for (int i = 0; i < CT_W; ++i)
#pragma unroll
                for (int j = 0; j < RT_W; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        bf16x4 q;
#pragma unroll
                        for (int u = 0; u < 4; ++u) q[u] = (__bf16)(alpha * acc[i][j][4 * g + u]);
                        *(bf16x4*)(Xh + ((rt_base + j) * 32 + l32) * XP + (ct_base + i) * 32 + 8 * g + 4 * h) = q;
                    }
        }
        __syncthreads();
        }   // halves
        load_v(va, ct0);
        load_w(wa, ct0, 0);

        // ---- stream
        if constexpr (PIPE == 1) {
            VFrag vb2;
            Acc wb2;
            if constexpr (halves == 1) {
                for (int i = 0; i < nct; i += 2) {
                    if (i + 1 < nct) { load_v(vb2, ct0 + i + 1); load_w(wb2, ct0 + i + 1, 0); }
                    compute_store(va, wa, ct0 + i, 0, -1);
                    if (i + 1 < nct) {
                        if (i + 2 < nct) { load_v(va, ct0 + i + 2); load_w(wa, ct0 + i + 2, 0); }
                        compute_store(vb2, wb2, ct0 + i + 1, 0, -1);
                    }
                }
            } else {
                // sub-tiles (ct, upper half), (ct, lower half), (ct + 1, upper half), ...: W one
                // sub-tile ahead, V one column tile ahead
                for (int i = 0; i < nct; i += 2) {
                    load_w(wb2, ct0 + i, 1);
                    if (i + 1 < nct) load_v(vb2, ct0 + i + 1);
                    compute_store(va, wa, ct0 + i, 0, -1);
                    if (i + 1 < nct) load_w(wa, ct0 + i + 1, 0);
                    compute_store(va, wb2, ct0 + i, 1, -1);
                    if (i + 1 < nct) {
                        load_w(wb2, ct0 + i + 1, 1);
                        if (i + 2 < nct) load_v(va, ct0 + i + 2);
                        compute_store(vb2, wa, ct0 + i + 1, 0, -1);
                        if (i + 2 < nct) load_w(wa, ct0 + i + 2, 0);
                        compute_store(vb2, wb2, ct0 + i + 1, 1, -1);
                    }
                }
            }
        } else {
            Acc wb2;
            for (int i = 0; i < nct; i += 2) {
                if (i + 1 < nct) load_w(wb2, ct0 + i + 1, 0);
                compute_store(va, wa, ct0 + i, 0, (i + 1 < nct && !skip) ? ct0 + i + 1 : -1);
                if (i + 1 < nct) {
                    if (i + 2 < nct) load_w(wa, ct0 + i + 2, 0);
                    compute_store(va, wb2, ct0 + i + 1, 0, (i + 2 < nct && !skip) ? ct0 + i + 2 : -1);
                }
            }
        }
    }
}

// mode: 0 = 128-row items, in-place V prefetch, two workgroups per CU; 1 = 128-row items, software
// prefetch of whole tiles, one workgroup per CU; 2 = 256-row items, otherwise as 1
template <int KSTEPS>
static hipError_t launch_lift_r(const LiftBlock* blocks_dev, const LiftTile* tiles_dev, const LiftRange* ranges_dev,
                                int n_wgs, int mode, float alpha, float beta, hipStream_t stream) {
    typedef void (*fn_t)(const LiftBlock*, const LiftTile*, const LiftRange*, float, float);
    fn_t fn = (mode == 0) ? (fn_t)lift_kernel<KSTEPS, 2, 1, 2>
              : (mode == 1) ? (fn_t)lift_kernel<KSTEPS, 1, 1, 1> : (fn_t)lift_kernel<KSTEPS, 1, 2, 1>;
    const int lds = (mode == 2 ? 2 : 1) * LIFT_TM * (KSTEPS * 16 + 8) * 2;
    static thread_local const void* configured[16] = {nullptr};
    bool done = false;
    for (const void* c : configured) if (c == (const void*)fn) { done = true; break; }
    if (!done) {
        hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        for (const void*& c : configured) if (c == nullptr) { c = (const void*)fn; break; }
    }
    hipLaunchKernelGGL(fn, dim3(n_wgs), dim3(LIFT_THREADS), lds, stream, blocks_dev, tiles_dev, ranges_dev, alpha, beta);
    return hipGetLastError();
}

hipError_t launch_lift(const LiftBlock* blocks_dev, const LiftTile* tiles_dev, const LiftRange* ranges_dev, int n_wgs,
                       int r, int mode, float alpha, float beta, hipStream_t stream) {
    if (n_wgs <= 0) return hipSuccess;
    switch (r) {
        case 64: return launch_lift_r<4>(blocks_dev, tiles_dev, ranges_dev, n_wgs, mode, alpha, beta, stream);
        case 128: return launch_lift_r<8>(blocks_dev, tiles_dev, ranges_dev, n_wgs, mode, alpha, beta, stream);
        case 256: return launch_lift_r<16>(blocks_dev, tiles_dev, ranges_dev, n_wgs, mode, alpha, beta, stream);
        default: return hipErrorInvalidValue;
    }
}

bool lift_supports_rank(int r) { return r == 64 || r == 128 || r == 256; }
int lift_panel_rows(int mode) { return mode == 2 ? 2 * LIFT_TM : LIFT_TM; }
int lift_wgs_per_cu(int mode) { return mode == 0 ? 2 : 1; }

}  // namespace tsr
