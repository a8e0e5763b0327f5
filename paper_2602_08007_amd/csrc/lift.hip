// Fused back-projection + weight update for the bf16 step path on gfx950:
//     W <- beta W + alpha (U D) V^T           (alpha = -lr*scale, beta = 1 - lr*wd)
// One workgroup (4 waves) owns a 128-row panel of one block and a run of 128-column tiles.
//   setup : T = U_panel D (128 x r) is computed once with MFMAs (U panel staged in LDS, D^T
//           fragments straight from L2) and parked in LDS as bf16;
//   stream: each wave owns 32 of the tile's 128 columns.  Its V fragments (32 columns x r)
//           come straight from global memory in MFMA operand layout and its W values are
//           loaded in accumulator layout, both one tile ahead, so nothing but T touches LDS
//           and the streaming loop has no barriers.  W crosses HBM exactly once each way and
//           neither T nor U D V^T is ever written to memory.
// The k index of every MFMA is permuted (lane half h takes k in [h r/2, (h+1) r/2)) so that
// each lane's operand bytes are contiguous in memory; both operands use the same permutation.
#include "lift.h"

namespace tsr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int LIFT_THREADS = 256;

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
__device__ inline float buf_load32(rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}
__device__ inline void buf_store32(float v, rsrc_t r, unsigned voff, unsigned soff) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)voff, (int)soff, 0);
}

__device__ inline void buf_store128(u32x4 v, rsrc_t r, unsigned voff, unsigned soff) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)voff, (int)soff, 0);
}

// VEC4: W rows are 16-byte aligned and n % 4 == 0.  The stream phase then runs the MFMA with
// the roles swapped (V fragment as the row operand), which puts four consecutive W columns
// into four consecutive accumulator registers of a lane: every W access is a 16-byte vector
// and a tile costs 16 loads + 16 stores per lane instead of 64 + 64, which also keeps the
// count of outstanding memory operations low enough to wait on the older tile only.
// LIFT_TM: rows of the panel (128 or 64).  PIPE: prefetch the next tile's V fragments and W
// values while the current tile is multiplied (one workgroup per CU) instead of relying on
// several resident workgroups (MINB per CU) to hide the memory latency.
template <int KSTEPS, bool VEC4, int LIFT_TM, bool PIPE, int MINB>
__global__ __launch_bounds__(LIFT_THREADS, MINB) void lift_kernel(const LiftBlock* blocks, const LiftTile* tiles,
                                                                  const float alpha, const float beta) {
    constexpr int R = KSTEPS * 16;
    constexpr int XP = R + 8;                 // padded LDS row (bf16 elements)
    constexpr int NCT = R / 32;               // 32-wide column tiles of T
    constexpr int RT = LIFT_TM / 32;          // 32-row tiles of the panel
    constexpr int CT_W = (NCT >= 4) ? NCT / 4 : 1;            // T column tiles per wave (setup)
    constexpr int WAVES_PER_CT = (NCT >= 4) ? 1 : 4 / NCT;
    constexpr int RT_W = (RT / WAVES_PER_CT > 0) ? RT / WAVES_PER_CT : 1;   // T row tiles per wave (setup)
    static_assert(RT % WAVES_PER_CT == 0, "panel rows must split over the waves of a column tile");
    extern __shared__ __attribute__((aligned(16))) unsigned short X[];   // [LIFT_TM][XP]

    const LiftTile t = tiles[blockIdx.x];
    if (t.block < 0) return;
    const LiftBlock b = blocks[t.block];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int row0 = t.row0;

    const rsrc_t rU = make_rsrc(b.Ub, (long long)b.m * b.ldr * 2);
    const rsrc_t rD = make_rsrc(b.DTb, (long long)b.r * b.ldr * 2);
    const rsrc_t rV = make_rsrc(b.Vb, (long long)b.n * b.ldr * 2);
    const rsrc_t rW = make_rsrc(b.W, ((long long)(b.m - 1) * b.ldw + b.n) * 4);
    const unsigned ldr_b = (unsigned)b.ldr * 2u, ldw_b = (unsigned)b.ldw * 4u;

    // ---- setup 1: U panel -> LDS (rows beyond m read as zero)
    {
        constexpr int CPR = R / 8;                            // 16-byte chunks per row
        constexpr int PER_THREAD = LIFT_TM * CPR / LIFT_THREADS;
        constexpr int GRP = PER_THREAD < 8 ? PER_THREAD : 8;
#pragma unroll
        for (int g = 0; g < PER_THREAD; g += GRP) {
            u32x4 v[GRP];
#pragma unroll
            for (int u = 0; u < GRP; ++u) {
                const int c = tid + LIFT_THREADS * (g + u);
                const int row = c / CPR, kc = (c % CPR) * 8;
                v[u] = buf_load128(rU, (unsigned)(row0 + row) * ldr_b + kc * 2, 0);
            }
#pragma unroll
            for (int u = 0; u < GRP; ++u) {
                const int c = tid + LIFT_THREADS * (g + u);
                const int row = c / CPR, kc = (c % CPR) * 8;
                *(u32x4*)(X + row * XP + kc) = v[u];
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
            const int kofs = h * (R / 2) + s * 8;
            bf16x8 fd[CT_W], fu[RT_W];
#pragma unroll
            for (int i = 0; i < CT_W; ++i)
                fd[i] = __builtin_bit_cast(bf16x8, buf_load128(rD, (unsigned)((ct_base + i) * 32 + l32) * ldr_b + kofs * 2, 0));
#pragma unroll
            for (int j = 0; j < RT_W; ++j) fu[j] = *(const bf16x8*)(X + ((rt_base + j) * 32 + l32) * XP + kofs);
#pragma unroll
            for (int i = 0; i < CT_W; ++i)
#pragma unroll
                for (int j = 0; j < RT_W; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[i], fu[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();                                      // every wave is done reading U from X
        // acc element e of tile (ct, rt): T column c = ct*32 + 8*(e/4) + 4*h + e%4, T row = rt*32 + l32
#pragma unroll
        for (int i = 0; i < CT_W; ++i)
#pragma unroll
            for (int j = 0; j < RT_W; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 q;
#pragma unroll
                    for (int u = 0; u < 4; ++u) q[u] = (__bf16)acc[i][j][4 * g + u];
                    const int c0 = (ct_base + i) * 32 + 8 * g + 4 * h;
                    const int row = (rt_base + j) * 32 + l32;
                    *(bf16x4*)(X + row * XP + c0) = q;
                }
    }
    __syncthreads();

    // ---- stream: W tile columns col0 + wave*32 + l32
    // The W tile is loaded (one tile ahead) straight into the accumulator registers of the
    // tile it belongs to; before the MFMAs it is scaled by beta/alpha so that alpha * acc is the
    // updated tile.  alpha == 0 (zero learning rate) skips the products.
    struct VFrag { u32x4 v[KSTEPS]; };
    struct Acc { f32x16 a[RT]; };
    const bool skip = (alpha == 0.0f);
    const float in_scale = skip ? beta : beta / alpha;
    const float out_scale = skip ? 1.0f : alpha;
    auto load_v = [&](VFrag& f, int ct) {
        const unsigned col = ct * 128 + wave * 32 + l32;           // columns beyond n read as zero
        const unsigned voff = col * ldr_b + h * R;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) f.v[s] = buf_load128(rV, voff + s * 16, 0);
    };
    auto w_voff = [&](int ct) -> unsigned {
        if constexpr (VEC4) {
            const int col = ct * 128 + wave * 32 + 4 * h;          // + 8 g + u
            // guarded per 4-column group and row tile where it is used
            return (unsigned)(row0 + l32) * ldw_b + (unsigned)col * 4u;
        } else {
            const int col = ct * 128 + wave * 32 + l32;
            return (col < b.n) ? (unsigned)(row0 + h * 4) * ldw_b + (unsigned)col * 4u : OOB_LANE;
        }
    };
    auto load_w = [&](Acc& w, int ct) {
        const unsigned voff = w_voff(ct);
        if constexpr (VEC4) {
            const int colb = ct * 128 + wave * 32 + 4 * h;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const bool ok = (colb + 8 * g < b.n) && (row0 + rt * 32 + l32 < b.m);
                    const unsigned vo = ok ? voff : OOB_LANE;
                    // four dword loads at consecutive immediate offsets: merged into one dwordx4
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        w.a[rt][4 * g + u] = buf_load32(rW, vo + 4 * u, (unsigned)(rt * 32) * ldw_b + g * 32);
                }
        } else {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = rt * 32 + (e >> 2) * 8 + (e & 3);
                    w.a[rt][e] = buf_load32(rW, (row0 + h * 4 + dr < b.m) ? voff : OOB_LANE, (unsigned)dr * ldw_b);
                }
        }
    };
    auto compute_store = [&](const VFrag& f, Acc& w, int ct) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int e = 0; e < 16; ++e) w.a[rt][e] *= in_scale;
        if (!skip) {
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const int kofs = h * (R / 2) + s * 8;
                const bf16x8 fv = __builtin_bit_cast(bf16x8, f.v[s]);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const bf16x8 ft = *(const bf16x8*)(X + (rt * 32 + l32) * XP + kofs);
                    if constexpr (VEC4) w.a[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv, ft, w.a[rt], 0, 0, 0);
                    else w.a[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ft, fv, w.a[rt], 0, 0, 0);
                }
            }
        }
        const unsigned voff = w_voff(ct);
        if constexpr (VEC4) {
            const int colb = ct * 128 + wave * 32 + 4 * h;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const bool ok = (colb + 8 * g < b.n) && (row0 + rt * 32 + l32 < b.m);
                    const unsigned vo = ok ? voff : OOB_LANE;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        buf_store32(out_scale * w.a[rt][4 * g + u], rW, vo + 4 * u, (unsigned)(rt * 32) * ldw_b + g * 32);
                }
        } else {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = rt * 32 + (e >> 2) * 8 + (e & 3);
                    buf_store32(out_scale * w.a[rt][e], rW, (row0 + h * 4 + dr < b.m) ? voff : OOB_LANE, (unsigned)dr * ldw_b);
                }
        }
    };

    const int ct0 = t.ct0, nct = t.nct;
    if constexpr (PIPE) {
        VFrag va, vb2;
        Acc wa, wb2;
        load_v(va, ct0);
        load_w(wa, ct0);
        for (int i = 0; i < nct; i += 2) {
            if (i + 1 < nct) { load_v(vb2, ct0 + i + 1); load_w(wb2, ct0 + i + 1); }
            compute_store(va, wa, ct0 + i);
            if (i + 1 < nct) {
                if (i + 2 < nct) { load_v(va, ct0 + i + 2); load_w(wa, ct0 + i + 2); }
                compute_store(vb2, wb2, ct0 + i + 1);
            }
        }
    } else {
        VFrag va;
        Acc wa;
        for (int i = 0; i < nct; ++i) {
            load_v(va, ct0 + i);
            load_w(wa, ct0 + i);
            compute_store(va, wa, ct0 + i);
        }
    }
}

// vec4: every block of the launch has 16-byte aligned W rows and n % 4 == 0.
// mode: 0 = 128-row panels with software prefetch, 1 = 64-row panels, several workgroups per CU,
//       2 = 64-row panels with software prefetch
template <int KSTEPS>
static hipError_t launch_lift_r(const LiftBlock* blocks_dev, const LiftTile* tiles_dev, int n_tiles, bool vec4, int mode,
                                float alpha, float beta, hipStream_t stream) {
    typedef void (*fn_t)(const LiftBlock*, const LiftTile*, float, float);
    fn_t fn;
    int tm;
    if (mode == 1) { fn = vec4 ? lift_kernel<KSTEPS, true, 64, false, 3> : lift_kernel<KSTEPS, false, 64, false, 3>; tm = 64; }
    else if (mode == 2) { fn = vec4 ? lift_kernel<KSTEPS, true, 64, true, 2> : lift_kernel<KSTEPS, false, 64, true, 2>; tm = 64; }
    else { fn = vec4 ? lift_kernel<KSTEPS, true, 128, true, 1> : lift_kernel<KSTEPS, false, 128, true, 1>; tm = 128; }
    const int lds = tm * (KSTEPS * 16 + 8) * 2;
    static thread_local const void* configured[8] = {nullptr};
    bool done = false;
    for (const void* c : configured) if (c == (const void*)fn) { done = true; break; }
    if (!done) {
        hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        for (const void*& c : configured) if (c == nullptr) { c = (const void*)fn; break; }
    }
    hipLaunchKernelGGL(fn, dim3(n_tiles), dim3(LIFT_THREADS), lds, stream, blocks_dev, tiles_dev, alpha, beta);
    return hipGetLastError();
}

hipError_t launch_lift(const LiftBlock* blocks_dev, const LiftTile* tiles_dev, int n_tiles, int r, bool vec4, int mode,
                       float alpha, float beta, hipStream_t stream) {
    if (n_tiles <= 0) return hipSuccess;
    switch (r) {
        case 64: return launch_lift_r<4>(blocks_dev, tiles_dev, n_tiles, vec4, mode, alpha, beta, stream);
        case 128: return launch_lift_r<8>(blocks_dev, tiles_dev, n_tiles, vec4, mode, alpha, beta, stream);
        case 256: return launch_lift_r<16>(blocks_dev, tiles_dev, n_tiles, vec4, mode, alpha, beta, stream);
        default: return hipErrorInvalidValue;
    }
}

bool lift_supports_rank(int r) { return r == 64 || r == 128 || r == 256; }
int lift_panel_rows(int mode) { return mode == 0 ? 128 : 64; }

}  // namespace tsr
