// C ABI of the TSR-Adam library: argument validation, workspace carving, and the launch
// sequences that compose the per-step path and the randomized-SVD refresh out of the grouped
// GEMM family and the small kernels.  No device memory is allocated here: everything lives in
// the caller's buffers and workspace.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/tsr.h"
#include "gemm.h"
#include "small.h"
#include "nt_gemm.h"
#include "host_util.h"
#include "fast_step.h"

using namespace tsr;

namespace tsr {
int& last_hip_error() {
    static thread_local int e = 0;
    return e;
}
}  // namespace tsr

namespace {

// ------------------------------------------------------------------ GEMM stages
struct LogicalGemm {
    const void* A; const float* B;
    long long lda, ldb;
    int M, N, K;
    float* out; long long ldc;
    int group = -1;                // consecutive entries with the same group >= 0 are summed into `out`
};

struct GemmStage {
    GemmVariant var{};
    std::vector<GemmProblem> probs;
    std::vector<GemmTile> tiles;
    std::vector<ReduceProblem> reduces;
    int max_reduce_elems = 0;
    bool direct = true;
    int tiles_m = 0, tiles_n = 0, ksplit = 1;      // single-problem decode
    const GemmProblem* d_probs = nullptr;
    const GemmTile* d_tiles = nullptr;
    const ReduceProblem* d_reduces = nullptr;
    bool empty() const { return probs.empty(); }
};

// Decide k-splits, carve partial buffers from `ar`, and list the tiles.
// want_tiles: keep splitting k while the launch has fewer tiles than this.
// lower_only: the outputs are symmetric and only tiles on or below the diagonal are computed
// (the rest of the output is left unwritten).
void build_stage(GemmStage& st, const GemmVariant& var, const std::vector<LogicalGemm>& gemms, Arena& ar,
                 int want_tiles = 512, bool lower_only = false) {
    st = GemmStage{};
    st.var = var;
    if (gemms.empty()) return;
    long long base_tiles = 0;
    bool shared_out = false;
    for (size_t i = 0; i < gemms.size(); ++i) {
        base_tiles += (long long)ceil_div(gemms[i].M, GEMM_BM) * ceil_div(gemms[i].N, GEMM_BN);
        if (i > 0 && gemms[i].group >= 0 && gemms[i].group == gemms[i - 1].group) shared_out = true;
    }
    int want_split = (int)std::max<long long>(1, want_tiles / std::max<long long>(1, base_tiles));
    std::vector<int> ksplit(gemms.size()), kchunk(gemms.size());
    bool any_split = false;
    for (size_t i = 0; i < gemms.size(); ++i) {
        const int K = gemms[i].K;
        int s = std::min(want_split, std::max(1, K / 256));
        int chunk = ceil_div(ceil_div(K, s), 32) * 32;
        s = ceil_div(K, chunk);
        ksplit[i] = s; kchunk[i] = chunk;
        if (s > 1) any_split = true;
    }
    st.direct = !(any_split || shared_out);
    st.probs.resize(gemms.size());
    size_t i = 0;
    while (i < gemms.size()) {
        // [i, e) = consecutive gemms summed into one output; their partials are one buffer
        size_t e = i + 1;
        while (e < gemms.size() && gemms[i].group >= 0 && gemms[e].group == gemms[i].group) ++e;
        const size_t mn = (size_t)gemms[i].M * gemms[i].N;
        float* part = nullptr;
        int group_splits = 0;
        if (!st.direct) {
            for (size_t j = i; j < e; ++j) group_splits += ksplit[j];
            part = ar.take<float>(mn * group_splits);
            ReduceProblem r{};
            r.part = part; r.out = gemms[i].out; r.stride = (long long)mn; r.ldc = gemms[i].ldc;
            r.M = gemms[i].M; r.N = gemms[i].N; r.splits = group_splits;
            st.reduces.push_back(r);
            st.max_reduce_elems = std::max(st.max_reduce_elems, (int)std::min<size_t>(mn, 1u << 30));
        }
        int prefix = 0;
        for (size_t j = i; j < e; ++j) {
            const LogicalGemm& g = gemms[j];
            GemmProblem& p = st.probs[j];
            p.A = g.A; p.B = g.B; p.lda = g.lda; p.ldb = g.ldb;
            p.M = g.M; p.N = g.N; p.K = g.K;
            if (st.direct) {
                p.C = g.out; p.ldc = g.ldc; p.c_split_stride = 0;
                p.kchunk = std::max(32, ceil_div(g.K, 32) * 32);
                ksplit[j] = 1;
            } else {
                p.C = part ? part + mn * prefix : nullptr;
                p.ldc = g.N; p.c_split_stride = (long long)mn; p.kchunk = kchunk[j];
                prefix += ksplit[j];
            }
            const int tmn = ceil_div(g.M, GEMM_BM), tnn = ceil_div(g.N, GEMM_BN);
            for (int ks = 0; ks < ksplit[j]; ++ks)
                for (int tm = 0; tm < tmn; ++tm)
                    for (int tn = 0; tn < tnn; ++tn)
                        if (!lower_only || tn <= tm) st.tiles.push_back(GemmTile{(int)j, tm, tn, ks});
            st.tiles_m = tmn; st.tiles_n = tnn; st.ksplit = ksplit[j];
        }
        i = e;
    }
}

int run_stage(const GemmStage& st, bool grouped, float alpha, float beta, Ctx& cx, int kind) {
    if (st.empty()) return TSR_OK;
    Timed timed(cx, kind);
    hipStream_t stream = cx.s;
    GemmLaunch L{};
    L.n_tiles = (int)st.tiles.size();
    if (grouped) {
        L.probs = st.d_probs; L.tiles = st.d_tiles;
    } else {
        L.single = st.probs[0];
        L.tiles_m = st.tiles_m; L.tiles_n = st.tiles_n; L.ksplit = st.ksplit;
        L.n_tiles = st.tiles_m * st.tiles_n * st.ksplit;       // the block index is decoded over the full grid
    }
    if (st.direct) {
        L.alpha = alpha; L.beta = beta;
        TSR_HIP(launch_gemm(L, st.var, stream));
    } else {
        L.alpha = 1.0f; L.beta = 0.0f;
        TSR_HIP(launch_gemm(L, st.var, stream));
        TSR_HIP(launch_splitk_reduce(grouped ? st.d_reduces : nullptr, grouped ? nullptr : &st.reduces[0],
                                     (int)st.reduces.size(), st.max_reduce_elems, alpha, beta, stream));
    }
    return TSR_OK;
}

void upload_stage(GemmStage& st, Arena& ar, Uploader& up) {
    if (st.empty()) return;
    st.d_probs = up.put(st.probs, ar);
    st.d_tiles = up.put(st.tiles, ar);
    if (!st.direct) st.d_reduces = up.put(st.reduces, ar);
}

inline GemmVariant variant(int aks, int bks, int abf, int pa, int pb) {
    GemmVariant v; v.a_kstrided = aks; v.b_kstrided = bks; v.a_bf16 = abf; v.a_pieces = abf ? 1 : pa; v.b_pieces = pb;
    return v;
}

// ------------------------------------------------------------------ validation helpers
bool aligned256(const void* p) { return ((uintptr_t)p % ALIGN) == 0; }

int check_block(int m, int n, int r) {
    if (m <= 0 || n <= 0 || r <= 0) return TSR_BAD_SHAPE;
    if (r > m || r > n) return TSR_BAD_SHAPE;
    return TSR_OK;
}
int check_dtype(int d) { return (d == TSR_F32 || d == TSR_BF16) ? TSR_OK : TSR_BAD_DTYPE; }
int check_prec(int p) { return (p == TSR_PREC_SPLIT || p == TSR_PREC_BF16) ? TSR_OK : TSR_INVALID_ARG; }

// ------------------------------------------------------------------ per-step programs
struct ProjectProgram {
    GemmStage gv[2];        // P = G V, index = dtype of G
    GemmStage utp;          // C = U^T P (summed over workers and k-splits)
};

// P buffers: one m x r fp32 per (block, worker), carved from `ar`.
void build_project(ProjectProgram& pg, const std::vector<BlockView>& blocks, int n_workers, int prec, Arena& ar) {
    std::vector<LogicalGemm> gv[2], utp;
    int group = 0;
    for (const BlockView& b : blocks) {
        const int esz = (b.g_dtype == TSR_BF16) ? 2 : 4;
        ++group;
        for (int w = 0; w < n_workers; ++w) {
            float* P = ar.take<float>((size_t)b.m * b.r);
            const char* Gw = b.G ? (const char*)b.G + (size_t)w * b.g_stride * esz : nullptr;
            gv[b.g_dtype].push_back(LogicalGemm{Gw, b.V, b.ldg, b.r, b.m, b.r, b.n, P, b.r});
            utp.push_back(LogicalGemm{b.U, P, b.r, b.r, b.r, b.r, b.m, b.C, b.r, group});
        }
    }
    const int pv = (prec == TSR_PREC_BF16) ? 1 : 2;
    build_stage(pg.gv[TSR_F32], variant(0, 1, 0, pv, pv), gv[TSR_F32], ar);
    build_stage(pg.gv[TSR_BF16], variant(0, 1, 1, 1, pv), gv[TSR_BF16], ar);
    build_stage(pg.utp, variant(1, 1, 0, pv, pv), utp, ar);
}

int run_project(const ProjectProgram& pg, bool grouped, float alpha, float beta, Ctx& cx) {
    TSR_TRY(run_stage(pg.gv[TSR_F32], grouped, 1.0f, 0.0f, cx, TSR_PROF_GV));
    TSR_TRY(run_stage(pg.gv[TSR_BF16], grouped, 1.0f, 0.0f, cx, TSR_PROF_GV));
    return run_stage(pg.utp, grouped, alpha, beta, cx, TSR_PROF_UTP);
}

struct LiftProgram {
    GemmStage ud;           // T = U D
    GemmStage tvt;          // W = beta W + alpha T V^T
};

void build_lift(LiftProgram& lp, const std::vector<BlockView>& blocks, int prec, Arena& ar) {
    std::vector<LogicalGemm> ud, tvt;
    for (const BlockView& b : blocks) {
        float* T = ar.take<float>((size_t)b.m * b.r);
        ud.push_back(LogicalGemm{b.U, b.D, b.r, b.r, b.m, b.r, b.r, T, b.r});
        tvt.push_back(LogicalGemm{T, b.V, b.r, b.r, b.m, b.n, b.r, b.W, b.ldw});
    }
    const int pv = (prec == TSR_PREC_BF16) ? 1 : 2;
    build_stage(lp.ud, variant(0, 1, 0, pv, pv), ud, ar, /*want_tiles=*/1);
    build_stage(lp.tvt, variant(0, 0, 0, pv, pv), tvt, ar, /*want_tiles=*/1);
}

int run_lift(const LiftProgram& lp, bool grouped, float lr, float wd, float scale, Ctx& cx) {
    TSR_TRY(run_stage(lp.ud, grouped, 1.0f, 0.0f, cx, TSR_PROF_UD));
    // W - lr (scale dW + wd W) = (1 - lr wd) W + (-lr scale) dW
    return run_stage(lp.tvt, grouped, -lr * scale, 1.0f - lr * wd, cx, TSR_PROF_TVT);
}

// ------------------------------------------------------------------ refresh program
struct RefreshBlock {
    const void* G; int g_dtype; int m, n, r, k; long long ldg;
    float* U; float* V; float* sigma;
    // workspace
    float *Y, *Yalt, *Z, *Zalt, *S, *Rinv, *XrT, *GrT;
    double *work, *R1, *Rmid, *Rtot, *Gacc, *eig;
    // bf16 gradients of a plan: the products with G on the k-contiguous bf16 family (see NtRefresh)
    bool nt = false;
    unsigned short *Gt = nullptr, *Pn = nullptr, *Pm = nullptr;   // G^T (n x ldm); pieces of a k x n / k x m operand
    unsigned short *Xp = nullptr, *Rt = nullptr;                  // pieces of a sketch (rows x ldk) and of R^-T (k x ldk)
    long long ldm = 0, ldn = 0, ldk = 0;
};

// orth(X) for X (rows x k) by Cholesky QR; the result is always left in Xalt (X is scratch).
//   passes = 1 (normalisations inside the power iteration): one SHIFTED pass, Xalt = X R^-1 with
//     R^T R = X^T X + s I.  Same span and the same triangular orientation as the exact factor; the
//     shift keeps the factorization from breaking down however ill conditioned the sketch is (a
//     steep spectrum squares into a Gram matrix whose small eigenvalues lie below its fp32-grade
//     rounding), at the price of a basis that is only roughly orthonormal, which is all these
//     intermediate bases are for.
//   passes = 3 (the final Q and the factor of B^T): shifted pass A (X -> Xalt), shifted pass E
//     (Xalt -> X), plain pass B with the Gram matrix at three bf16 pieces (X -> Xalt).  Each
//     shifted pass brings the condition number down to about 1 / sqrt(shift) of what it was, so
//     sketches with a condition number up to about 1e6 arrive at pass B well conditioned; pass B
//     drops what is left at rounding level (pivot <= 1e-6 of its diagonal entry: directions beyond
//     the numerical rank, e.g. of an exactly low-rank or zero gradient) as zero columns.
constexpr double ORTH_SHIFT = 1e-4;       // relative to the largest diagonal entry of the Gram matrix
constexpr double ORTH_DROP = 1e-6;

// A shifted pass (A or E) of the blocks with RefreshBlock::nt on the bf16 NT family.  The sketch X
// enters as two bf16 pieces in both orientations (transposed for the Gram matrix, as stored for the
// product with R^-1), R^-1 as two pieces of its transpose; every product keeps the three leading
// cross terms: X^T X = Xh^T Xh + Xl^T Xh + Xh^T Xl (summed by the k-split reduction, lower tiles
// only); X R^-1 as ONE product over a doubled contraction: the rows [Xh | Xl] against the two pieces
// [Rh | Rh] and [Rl | Rl] of the transposed factor, i.e. (Xh + Xl)(Rh + Rl).
struct OrthNtPass {
    std::vector<SplitBlock> st, sx, sr, sr2;  // X -> pieces of X^T; X -> [Xh | Xl]; R^-1 -> the two halves of the pieces of R^-T
    const SplitBlock* d_st = nullptr; const SplitBlock* d_sx = nullptr; const SplitBlock* d_sr = nullptr;
    const SplitBlock* d_sr2 = nullptr;
    NtStageH gram, ap;
    int max_rows = 0, max_k = 0;
    bool empty() const { return st.empty(); }
};

struct OrthProgram {
    OrthNtPass ntA, ntE;
    GemmStage gramA, qA, gramE, qE, gramB, qB;
    std::vector<CholBlock> cholA, cholE, cholB;
    const CholBlock* d_cholA = nullptr; const CholBlock* d_cholE = nullptr; const CholBlock* d_cholB = nullptr;
};

// The products with a bf16 gradient (Y = G Omega, Z = G^T Q, Y = G Qrow: Algorithm 1's sketch,
// power-iteration and B lines) in the operand form of the bf16 NT family, C = A B^T with both
// operands k-contiguous: A is the gradient itself, or a transposed copy made once per refresh; B is
// the transpose of the small fp32 operand cut into two bf16 pieces (written by a split kernel before
// each product), which the kernel multiplies with the same staged A tile.  The gradient is exact in
// bf16, so the product is accurate to the two pieces of the small operand (2^-18 per element), as on
// the general kernel.  One stage serves both products with G (their B pieces share a buffer).
constexpr int NT_REFRESH_PIECES = 2;
struct NtRefresh {
    std::vector<TransposeBlock> gt;   const TransposeBlock* d_gt = nullptr;
    std::vector<SplitBlock> s_om, s_q, s_qrow;
    const SplitBlock* d_om = nullptr; const SplitBlock* d_q = nullptr; const SplitBlock* d_qrow = nullptr;
    NtStageH g_stage, gt_stage;       // (m x k) = G (pieces over n)^T ; (n x k) = G^T (pieces over m)^T
    int max_m = 0, max_n = 0, max_k = 0;
    bool empty() const { return gt.empty(); }
};

struct RefreshProgram {
    std::vector<RefreshBlock> blocks;
    NtRefresh nt;           // blocks with RefreshBlock::nt; the GemmStages below hold the others
    GemmStage sketch[2];    // Y = G Omega
    GemmStage gtq[2];       // Z = G^T Q    (Q = orth result, held in Yalt)
    GemmStage gq[2];        // Y = G Qrow   (Qrow = orth result, held in Zalt)
    OrthProgram orthY, orthZ;
    std::vector<JacobiBlock> jac, jac_pre;
    const JacobiBlock* d_jac = nullptr; const JacobiBlock* d_jac_pre = nullptr;
    GemmStage uout, vout;
};

void build_orth_nt(OrthNtPass& pass, const std::vector<RefreshBlock>& blocks, bool on_rows_m, bool from_alt, Arena& ar) {
    pass = OrthNtPass{};
    std::vector<NtLogical> g, a1;
    for (size_t i = 0; i < blocks.size(); ++i) {
        const RefreshBlock& b = blocks[i];
        if (!b.nt) continue;
        const int rows = on_rows_m ? b.m : b.n, k = b.k;
        float* X = on_rows_m ? b.Y : b.Z;
        float* Xalt = on_rows_m ? b.Yalt : b.Zalt;
        const float* in = from_alt ? Xalt : X;
        float* out = from_alt ? X : Xalt;
        unsigned short* Xt = on_rows_m ? b.Pm : b.Pn;            // pieces of X^T (k x ldrows)
        const long long ldrows = on_rows_m ? b.ldm : b.ldn, st_t = (long long)k * ldrows;
        const long long ld2 = 2 * b.ldk, st_r = (long long)k * ld2;      // rows of two pieces side by side
        pass.st.push_back(SplitBlock{in, Xt, ldrows, st_t, rows, k});
        pass.sx.push_back(SplitBlock{in, b.Xp, ld2, b.ldk, rows, k});
        pass.sr.push_back(SplitBlock{b.Rinv, b.Rt, ld2, st_r, k, k});
        pass.sr2.push_back(SplitBlock{b.Rinv, b.Rt + b.ldk, ld2, st_r, k, k});
        const int bi = (int)i;
        g.push_back(NtLogical{Xt, Xt, b.S, ldrows, ldrows, k, k, k, rows, bi, bi});
        g.push_back(NtLogical{Xt + st_t, Xt, b.S, ldrows, ldrows, k, k, k, rows, bi, bi});
        g.push_back(NtLogical{Xt, Xt + st_t, b.S, ldrows, ldrows, k, k, k, rows, bi, bi});
        a1.push_back(NtLogical{b.Xp, b.Rt, out, ld2, ld2, k, rows, k, (int)ld2, bi, -1, st_r});
        pass.max_rows = std::max(pass.max_rows, rows); pass.max_k = std::max(pass.max_k, k);
    }
    if (g.empty()) return;
    const int nb = (int)blocks.size();
    build_nt_stage(pass.gram, NtVariant{NT_128x128, 0, 0}, g, nb, ar, 512, false, 0, /*lower_only=*/true);
    NtVariant v2{};
    const char* e = getenv("TSR_TUNE_ORTH_WIDE");          // 0: 128 x 128 tiles instead of the wide-tile kernel
    v2.shape = (e && e[0] == '0') ? (int)NT_128x128_K32 : (int)NT_256x128_K32; v2.b_pieces = 2;
    build_nt_stage(pass.ap, v2, a1, nb, ar, 1);
}

void build_orth(OrthProgram& op, const std::vector<RefreshBlock>& blocks, bool on_rows_m, Arena& ar) {
    std::vector<LogicalGemm> gA, qA, gE, qE, gB, qB;
    op.cholA.clear(); op.cholE.clear(); op.cholB.clear();
    const char* e = getenv("TSR_TUNE_ORTH_NT");            // 0: the shifted passes of every block on the general kernel
    const bool orth_nt = !(e && e[0] == '0');
    for (const RefreshBlock& b : blocks) {
        const int rows = on_rows_m ? b.m : b.n;
        float* X = on_rows_m ? b.Y : b.Z;
        float* Xalt = on_rows_m ? b.Yalt : b.Zalt;
        const int k = b.k;
        if (!(b.nt && orth_nt)) {
            gA.push_back(LogicalGemm{X, X, k, k, k, k, rows, b.S, k});
            qA.push_back(LogicalGemm{X, b.Rinv, k, k, rows, k, k, Xalt, k});
            gE.push_back(LogicalGemm{Xalt, Xalt, k, k, k, k, rows, b.S, k});
            qE.push_back(LogicalGemm{Xalt, b.Rinv, k, k, rows, k, k, X, k});
        }
        gB.push_back(LogicalGemm{X, X, k, k, k, k, rows, b.S, k});
        qB.push_back(LogicalGemm{X, b.Rinv, k, k, rows, k, k, Xalt, k});
        // the three triangular factors (X = Q R3 R2 R1) go to R1, Rmid and Gacc (free until the small
        // SVD); where their product is needed, fp64 MFMA GEMMs form it afterwards (run_refresh_back)
        op.cholA.push_back(CholBlock{b.S, b.Rinv, b.R1, b.work, k});
        op.cholE.push_back(CholBlock{b.S, b.Rinv, b.Rmid, b.work, k});
        op.cholB.push_back(CholBlock{b.S, b.Rinv, b.Gacc, b.work, k});
    }
    if (orth_nt) {
        build_orth_nt(op.ntA, blocks, on_rows_m, false, ar);
        build_orth_nt(op.ntE, blocks, on_rows_m, true, ar);
    } else {
        op.ntA = OrthNtPass{}; op.ntE = OrthNtPass{};
    }
    // The first pass meets the sketch at its raw scaling, where a rounding of X moves the span of
    // the result: with an fp32 gradient X keeps three bf16 pieces there, as in the products with G.
    int pieces_x = 2;
    for (const RefreshBlock& b : blocks) if (b.g_dtype == TSR_F32) pieces_x = 3;
    // the Cholesky kernels read the lower triangle of the Gram matrix only
    build_stage(op.gramA, variant(1, 1, 0, 2, 2), gA, ar, 512, true);
    build_stage(op.qA, variant(0, 1, 0, pieces_x, pieces_x), qA, ar, 1);
    build_stage(op.gramE, variant(1, 1, 0, 2, 2), gE, ar, 512, true);
    build_stage(op.qE, variant(0, 1, 0, 2, 2), qE, ar, 1);
    build_stage(op.gramB, variant(1, 1, 0, 3, 3), gB, ar, 512, true);
    build_stage(op.qB, variant(0, 1, 0, 3, 3), qB, ar, 1);
}

int run_orth(const OrthProgram& op, bool grouped, Ctx& cx, int passes) {
    const int nb = (int)op.cholA.size();
    int max_k = 0;
    for (const CholBlock& cb : op.cholA) max_k = std::max(max_k, cb.k);
    auto chol = [&](const CholBlock* dev, const std::vector<CholBlock>& host, double tol, double shift) -> int {
        Timed timed(cx, TSR_PROF_CHOL);
        TSR_HIP(launch_chol_inv(grouped ? dev : nullptr, grouped ? nullptr : &host[0], nb, max_k, tol, shift, cx.s));
        return TSR_OK;
    };
    // a shifted pass: Gram matrices (NT family for the blocks it takes, general kernel for the rest),
    // Cholesky of all of them, then the products with R^-1
    auto nt_gram = [&](const OrthNtPass& p) -> int {
        if (p.empty()) return TSR_OK;
        {
            Timed timed(cx, TSR_PROF_ORTH_GEMM);
            TSR_HIP(launch_split_transpose(p.d_st, (int)p.st.size(), p.max_rows, p.max_k, 2, cx.s));
        }
        return run_nt_stage(p.gram, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM);
    };
    auto nt_apply = [&](const OrthNtPass& p) -> int {
        if (p.empty()) return TSR_OK;
        {
            Timed timed(cx, TSR_PROF_ORTH_GEMM);
            TSR_HIP(launch_split_rows(p.d_sx, (int)p.sx.size(), p.max_rows, p.max_k, 2, cx.s));
            TSR_HIP(launch_split_transpose(p.d_sr, (int)p.sr.size(), p.max_k, p.max_k, 2, cx.s));
            TSR_HIP(launch_split_transpose(p.d_sr2, (int)p.sr2.size(), p.max_k, p.max_k, 2, cx.s));
        }
        return run_nt_stage(p.ap, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM);
    };
    TSR_TRY(nt_gram(op.ntA));
    TSR_TRY(run_stage(op.gramA, grouped, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM));
    TSR_TRY(chol(op.d_cholA, op.cholA, ORTH_DROP, ORTH_SHIFT));
    TSR_TRY(nt_apply(op.ntA));
    TSR_TRY(run_stage(op.qA, grouped, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM));
    if (passes == 1) return TSR_OK;
    TSR_TRY(nt_gram(op.ntE));
    TSR_TRY(run_stage(op.gramE, grouped, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM));
    TSR_TRY(chol(op.d_cholE, op.cholE, ORTH_DROP, ORTH_SHIFT));
    TSR_TRY(nt_apply(op.ntE));
    TSR_TRY(run_stage(op.qE, grouped, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM));
    TSR_TRY(run_stage(op.gramB, grouped, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM));
    TSR_TRY(chol(op.d_cholB, op.cholB, ORTH_DROP, 0.0));
    return run_stage(op.qB, grouped, 1.0f, 0.0f, cx, TSR_PROF_ORTH_GEMM);
}

void build_refresh_stages(RefreshProgram& rp, const float* const* omegas, Arena& ar);

// A bf16 gradient the NT family can read: 16-byte aligned base and rows, a row pitch that covers the
// width rounded up to 8 elements, every operand addressable with 31-bit byte offsets.
bool nt_refresh_eligible(const BlockView& v, int k) {
    const char* e = getenv("TSR_TUNE_REFRESH_NT");         // read when a plan is built
    if ((e && e[0] == '0') || v.g_dtype != TSR_BF16) return false;
    if (((uintptr_t)v.G) % 16 != 0 || (v.ldg * 2) % 16 != 0 || v.ldg < (v.n + 7) / 8 * 8) return false;
    const long long lim = 1LL << 31, big = std::max(v.m, v.n);
    if ((long long)(v.m + 256) * v.ldg * 2 >= lim) return false;                 // G
    if ((long long)(v.n + 256) * ((v.m + 7) / 8 * 8) * 2 >= lim) return false;   // G^T
    if ((long long)NT_REFRESH_PIECES * (k + 256) * ((big + 7) / 8 * 8) * 2 >= lim) return false;   // pieces
    if ((big + 256) * (long long)k * 4 >= lim) return false;                     // fp32 outputs
    return true;
}

// Carves every refresh buffer from `ar` and builds all stages.  Omega pointers may be null
// at build time (they are patched in before the launch).
void build_refresh(RefreshProgram& rp, const std::vector<BlockView>& views, const float* const* omegas, int p,
                   float* const* sigmas, Arena& ar, bool allow_nt = false) {
    rp.blocks.clear();
    for (size_t i = 0; i < views.size(); ++i) {
        const BlockView& v = views[i];
        RefreshBlock b{};
        b.G = v.G; b.g_dtype = v.g_dtype; b.m = v.m; b.n = v.n; b.r = v.r; b.k = v.r + p; b.ldg = v.ldg;
        b.U = v.U; b.V = v.V; b.sigma = sigmas ? sigmas[i] : nullptr;
        const size_t k = (size_t)b.k;
        b.Y = ar.take<float>((size_t)b.m * k); b.Yalt = ar.take<float>((size_t)b.m * k);
        b.Z = ar.take<float>((size_t)b.n * k); b.Zalt = ar.take<float>((size_t)b.n * k);
        b.S = ar.take<float>(k * k); b.Rinv = ar.take<float>(k * k);
        b.XrT = ar.take<float>((size_t)b.r * k); b.GrT = ar.take<float>((size_t)b.r * k);
        b.work = ar.take<double>(2 * k * k + 64); b.R1 = ar.take<double>(k * k); b.Rmid = ar.take<double>(k * k);
        b.Rtot = ar.take<double>(k * k); b.Gacc = ar.take<double>(k * k);
        b.eig = (b.k <= EIG_MAXK) ? ar.take<double>(3 * k * k + 3 * k + 8) : nullptr;
        if (allow_nt && nt_refresh_eligible(v, b.k)) {
            b.nt = true;
            b.ldm = (b.m + 7) / 8 * 8; b.ldn = (b.n + 7) / 8 * 8;
            b.Gt = ar.take<unsigned short>((size_t)b.n * b.ldm);
            b.Pn = ar.take<unsigned short>((size_t)NT_REFRESH_PIECES * k * b.ldn);
            b.Pm = ar.take<unsigned short>((size_t)NT_REFRESH_PIECES * k * b.ldm);
            b.ldk = (b.k + 7) / 8 * 8;
            b.Xp = ar.take<unsigned short>((size_t)NT_REFRESH_PIECES * std::max(b.m, b.n) * b.ldk);
            b.Rt = ar.take<unsigned short>((size_t)NT_REFRESH_PIECES * k * 2 * b.ldk);       // each piece twice, side by side
        }
        rp.blocks.push_back(b);
    }
    build_refresh_stages(rp, omegas, ar);
}

// Stages and tables of the refresh of rp.blocks (whose buffers are already carved).
void build_refresh_stages(RefreshProgram& rp, const float* const* omegas, Arena& ar) {
    std::vector<LogicalGemm> sk[2], gtq[2], gq[2], uo, vo;
    std::vector<NtLogical> ntg, ntgt;
    rp.nt = NtRefresh{};
    rp.jac.clear(); rp.jac_pre.clear();
    for (size_t i = 0; i < rp.blocks.size(); ++i) {
        const RefreshBlock& b = rp.blocks[i];
        const float* om = omegas ? omegas[i] : nullptr;
        if (b.nt) {
            NtRefresh& f = rp.nt;
            const long long sn = (long long)b.k * b.ldn, sm = (long long)b.k * b.ldm;
            f.gt.push_back(TransposeBlock{b.G, b.Gt, b.ldg, b.ldm, b.m, b.n});
            f.s_om.push_back(SplitBlock{om, b.Pn, b.ldn, sn, b.n, b.k});
            f.s_qrow.push_back(SplitBlock{b.Zalt, b.Pn, b.ldn, sn, b.n, b.k});
            f.s_q.push_back(SplitBlock{b.Yalt, b.Pm, b.ldm, sm, b.m, b.k});
            ntg.push_back(NtLogical{b.G, b.Pn, b.Y, b.ldg, b.ldn, b.k, b.m, b.k, b.n, (int)i, -1, sn});
            ntgt.push_back(NtLogical{b.Gt, b.Pm, b.Z, b.ldm, b.ldm, b.k, b.n, b.k, b.m, (int)i, -1, sm});
            f.max_m = std::max(f.max_m, b.m); f.max_n = std::max(f.max_n, b.n); f.max_k = std::max(f.max_k, b.k);
        } else {
            sk[b.g_dtype].push_back(LogicalGemm{b.G, om, b.ldg, b.k, b.m, b.k, b.n, b.Y, b.k});
            gtq[b.g_dtype].push_back(LogicalGemm{b.G, b.Yalt, b.ldg, b.k, b.n, b.k, b.m, b.Z, b.k});
            gq[b.g_dtype].push_back(LogicalGemm{b.G, b.Zalt, b.ldg, b.k, b.m, b.k, b.n, b.Y, b.k});
        }
        uo.push_back(LogicalGemm{b.Yalt, b.XrT, b.k, b.k, b.m, b.r, b.k, b.U, b.r});
        vo.push_back(LogicalGemm{b.Zalt, b.GrT, b.k, b.k, b.n, b.r, b.k, b.V, b.r});
        // R = R3 (R2 R1): first R2 R1 into the (by then idle) Cholesky work area, then the small SVD's
        // table with that product in the place of R1
        rp.jac_pre.push_back(JacobiBlock{b.work, b.Rmid, nullptr, nullptr, nullptr, nullptr, b.k, b.r, nullptr, b.R1});
        rp.jac.push_back(JacobiBlock{b.Rtot, b.Gacc, b.work, b.XrT, b.GrT, b.sigma, b.k, b.r, b.eig, b.work});
    }
    for (int d = 0; d < 2; ++d) {
        // an fp32 gradient keeps three bf16 pieces per operand (rounding at 2^-27, below its own
        // 2^-24); a bf16 gradient is exact in one piece and meets the sketch at two pieces
        const int pc = (d == TSR_F32) ? 3 : 2;
        build_stage(rp.sketch[d], variant(0, 1, d, pc, pc), sk[d], ar);
        build_stage(rp.gtq[d], variant(1, 1, d, pc, pc), gtq[d], ar);
        build_stage(rp.gq[d], variant(0, 1, d, pc, pc), gq[d], ar);
    }
    {
        // the wide-tile kernel (256 x 128 outputs, two pieces of B); TSR_TUNE_REFRESH_WIDE=0: 128 x 128 tiles,
        // two workgroups per compute unit (measured on the 1B workload: 23.2 against 26.0 ms, equal on the 130M one)
        const char* e = getenv("TSR_TUNE_REFRESH_WIDE");
        NtVariant var{};
        var.shape = (e && e[0] == '0') ? (int)NT_128x128_K32 : (int)NT_256x128_K32; var.b_pieces = NT_REFRESH_PIECES;
        build_nt_stage(rp.nt.g_stage, var, ntg, (int)rp.blocks.size(), ar, 512);
        build_nt_stage(rp.nt.gt_stage, var, ntgt, (int)rp.blocks.size(), ar, 512);
    }
    build_orth(rp.orthY, rp.blocks, true, ar);
    build_orth(rp.orthZ, rp.blocks, false, ar);
    build_stage(rp.uout, variant(0, 0, 0, 3, 3), uo, ar, 1);
    build_stage(rp.vout, variant(0, 0, 0, 3, 3), vo, ar, 1);
}

// Sketch chain of one worker: leaves the final Q in Yalt and B^T = G^T Q in Z.  Inside the power
// iteration the bases are normalised by one shifted Cholesky pass (run_orth, passes = 1), the final
// Q by three: right-multiplying a sketch by an upper-triangular factor changes neither its span nor
// the Q factor of anything computed from it.
int run_refresh_front(const RefreshProgram& rp, bool grouped, int q, Ctx& cx) {
    const NtRefresh& f = rp.nt;
    const bool nt = !f.empty();           // only in programs with device tables (grouped)
    // a product with G or G^T on the NT family: the small operand cut into pieces, then the GEMM
    auto nt_product = [&](const SplitBlock* split, const NtStageH& stage, int rows) -> int {
        if (!nt) return TSR_OK;
        {
            Timed timed(cx, TSR_PROF_SKETCH_GEMM);
            TSR_HIP(launch_split_transpose(split, (int)f.gt.size(), rows, f.max_k, NT_REFRESH_PIECES, cx.s));
        }
        return run_nt_stage(stage, 1.0f, 0.0f, cx, TSR_PROF_SKETCH_GEMM);
    };
    if (nt) {
        Timed timed(cx, TSR_PROF_SKETCH_GEMM);
        TSR_HIP(launch_transpose_bf16(f.d_gt, (int)f.gt.size(), f.max_m, f.max_n, cx.s));
    }
    TSR_TRY(nt_product(f.d_om, f.g_stage, f.max_n));
    for (int d = 0; d < 2; ++d) TSR_TRY(run_stage(rp.sketch[d], grouped, 1.0f, 0.0f, cx, TSR_PROF_SKETCH_GEMM));
    for (int it = 0; it < q; ++it) {
        TSR_TRY(run_orth(rp.orthY, grouped, cx, 1));                                    // Q' in Yalt
        TSR_TRY(nt_product(f.d_q, f.gt_stage, f.max_m));
        for (int d = 0; d < 2; ++d) TSR_TRY(run_stage(rp.gtq[d], grouped, 1.0f, 0.0f, cx, TSR_PROF_SKETCH_GEMM));
        TSR_TRY(run_orth(rp.orthZ, grouped, cx, 1));                                    // Q'row in Zalt
        TSR_TRY(nt_product(f.d_qrow, f.g_stage, f.max_n));
        for (int d = 0; d < 2; ++d) TSR_TRY(run_stage(rp.gq[d], grouped, 1.0f, 0.0f, cx, TSR_PROF_SKETCH_GEMM));
    }
    TSR_TRY(run_orth(rp.orthY, grouped, cx, 3));                                        // Q in Yalt
    TSR_TRY(nt_product(f.d_q, f.gt_stage, f.max_m));
    for (int d = 0; d < 2; ++d) TSR_TRY(run_stage(rp.gtq[d], grouped, 1.0f, 0.0f, cx, TSR_PROF_SKETCH_GEMM));
    return TSR_OK;
}

// From Q (in Yalt) and B^T (in Z):  B^T = Q_B R (Q_B in Zalt) ; SVD of R ; U = Q X_r ; V = Q_B Gacc_r^T
int run_refresh_back(const RefreshProgram& rp, bool grouped, Ctx& cx) {
    TSR_TRY(run_orth(rp.orthZ, grouped, cx, 3));
    {
        Timed timed(cx, TSR_PROF_JACOBI);
        int max_k = 0;
        for (const JacobiBlock& jb : rp.jac) max_k = std::max(max_k, jb.k);
        const int nb = (int)rp.jac.size();
        TSR_HIP(launch_rtot_product(grouped ? rp.d_jac_pre : nullptr, grouped ? nullptr : &rp.jac_pre[0], nb, max_k, cx.s));
        TSR_HIP(launch_rtot_product(grouped ? rp.d_jac : nullptr, grouped ? nullptr : &rp.jac[0], nb, max_k, cx.s));
        static const bool chain = [] { const char* e = getenv("TSR_TUNE_EIG_CHAIN"); return !(e && e[0] == '0'); }();
        if (chain && max_k <= EIG_MAXK)
            TSR_HIP(launch_eig_svd(grouped ? rp.d_jac : nullptr, grouped ? nullptr : &rp.jac[0], nb, max_k, cx.s));
        else
            TSR_HIP(launch_jacobi(grouped ? rp.d_jac : nullptr, grouped ? nullptr : &rp.jac[0], nb, max_k, cx.s));
    }
    TSR_TRY(run_stage(rp.uout, grouped, 1.0f, 0.0f, cx, TSR_PROF_BASIS_GEMM));
    return run_stage(rp.vout, grouped, 1.0f, 0.0f, cx, TSR_PROF_BASIS_GEMM);
}

int run_refresh(const RefreshProgram& rp, bool grouped, int q, Ctx& cx) {
    TSR_TRY(run_refresh_front(rp, grouped, q, cx));
    return run_refresh_back(rp, grouped, cx);
}

int check_refresh_shape(int m, int n, int r, int p) {
    TSR_TRY(check_block(m, n, r));
    if (p < 0) return TSR_BAD_SHAPE;
    if ((long long)r + p > m || (long long)r + p > n) return TSR_BAD_SHAPE;
    if (r + p > 1024) return TSR_BAD_SHAPE;     // limit of the one-workgroup factorization kernels
    return TSR_OK;
}

}  // namespace

void upload_refresh(RefreshProgram& rp, Arena& ar, Uploader& up) {
    for (int d = 0; d < 2; ++d) {
        upload_stage(rp.sketch[d], ar, up); upload_stage(rp.gtq[d], ar, up); upload_stage(rp.gq[d], ar, up);
    }
    for (OrthProgram* op : {&rp.orthY, &rp.orthZ}) {
        for (OrthNtPass* p : {&op->ntA, &op->ntE}) {
            if (p->empty()) continue;
            p->d_st = up.put(p->st, ar); p->d_sx = up.put(p->sx, ar); p->d_sr = up.put(p->sr, ar); p->d_sr2 = up.put(p->sr2, ar);
            upload_nt_stage(p->gram, ar, up); upload_nt_stage(p->ap, ar, up);
        }
        upload_stage(op->gramA, ar, up); upload_stage(op->qA, ar, up);
        upload_stage(op->gramE, ar, up); upload_stage(op->qE, ar, up);
        upload_stage(op->gramB, ar, up); upload_stage(op->qB, ar, up);
        op->d_cholA = up.put(op->cholA, ar); op->d_cholE = up.put(op->cholE, ar); op->d_cholB = up.put(op->cholB, ar);
    }
    rp.d_jac = up.put(rp.jac, ar);
    rp.d_jac_pre = up.put(rp.jac_pre, ar);
    if (!rp.nt.empty()) {
        NtRefresh& f = rp.nt;
        f.d_gt = up.put(f.gt, ar);
        f.d_om = up.put(f.s_om, ar); f.d_q = up.put(f.s_q, ar); f.d_qrow = up.put(f.s_qrow, ar);
        upload_nt_stage(f.g_stage, ar, up);
        upload_nt_stage(f.gt_stage, ar, up);
    }
    upload_stage(rp.uout, ar, up); upload_stage(rp.vout, ar, up);
}

// Number of block groups the batched refresh runs side by side, each on a stream of its own:
// the factorization kernels keep one workgroup per matrix busy for milliseconds, the GEMM
// stages of the other groups fill the rest of the chip meanwhile.
int refresh_group_count(int blocks) {
    const char* e = getenv("TSR_TUNE_REFRESH_GROUPS");
    int g = e ? atoi(e) : 3;
    g = std::max(1, std::min(g, 4));       // one stream per group: beyond the four hardware queues of a process they serialise
    while (g > 1 && blocks / g < 4) --g;
    return g;
}

// ====================================================================== C ABI
struct tsr_plan {
    std::vector<BlockView> blocks;
    int n_workers = 1, precision = 0, p = 0;
    bool with_refresh = false;
    ProjectProgram project;
    LiftProgram lift;
    FastStep fast;              // used instead of project / lift when precision == TSR_PREC_BF16
    bool use_fast = false;
    bool force_generic = false;   // sizing only: measure the generic programs
    std::vector<CoreBlock> cores; const CoreBlock* d_cores = nullptr; long long max_core = 0;
    RefreshProgram refresh;
    // the same refresh cut into groups of blocks (sharing the buffers of `refresh`), run on
    // side streams when no stage timing is asked for
    std::vector<RefreshProgram> groups;
    std::vector<std::vector<int>> group_blocks;     // indices into refresh.blocks
    std::vector<hipStream_t> side;                  // groups 1.. (group 0 runs on the caller's stream)
    std::vector<hipEvent_t> joined;
    hipEvent_t fork = nullptr;
    char* ws = nullptr;
    Uploader up;
    Prof prof;
    ~tsr_plan() {
        prof.clear();
        for (hipStream_t st : side) (void)hipStreamDestroy(st);
        for (hipEvent_t ev : joined) (void)hipEventDestroy(ev);
        if (fork) (void)hipEventDestroy(fork);
    }
};

extern "C" {

const char* tsr_status_string(int status) {
    switch (status) {
        case TSR_OK: return "ok";
        case TSR_INVALID_ARG: return "invalid argument";
        case TSR_BAD_SHAPE: return "bad shape";
        case TSR_BAD_DTYPE: return "bad dtype";
        case TSR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case TSR_HIP_ERROR: return "HIP runtime error";
        case TSR_STATIC_SCRATCH_TOO_SMALL: return "problem needs more scratch than the built-in static buffer holds";
        default: return "unknown status";
    }
}

int tsr_last_hip_error(void) { return tsr::last_hip_error(); }

int tsr_device_count(void) {
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess) return 0;
    return n;
}

// ---------------------------------------------------------------- project
static void one_block_view(std::vector<BlockView>& v, const void* G, int g_dtype, int m, int n, int r,
                           long long ldg, float* W, long long ldw, float* U, float* V, float* C, float* D) {
    BlockView b{};
    b.G = G; b.g_dtype = g_dtype; b.m = m; b.n = n; b.r = r; b.ldg = ldg; b.g_stride = 0;
    b.W = W; b.ldw = ldw; b.U = U; b.V = V; b.C = C; b.D = D;
    v.assign(1, b);
}

size_t tsr_project_workspace_bytes(int m, int n, int r) {
    if (check_block(m, n, r) != TSR_OK) return 0;
    std::vector<BlockView> v;
    one_block_view(v, nullptr, TSR_F32, m, n, r, n, nullptr, n, nullptr, nullptr, nullptr, nullptr);
    Arena ar(nullptr);
    ProjectProgram pg;
    build_project(pg, v, 1, TSR_PREC_SPLIT, ar);
    return ar.used();
}

int tsr_project_core(const void* G, int g_dtype, int m, int n, long long ldg, const float* U, const float* V,
                     int r, float alpha, int accumulate, float* C, int precision, void* ws, size_t ws_bytes,
                     void* stream) {
    TSR_TRY(check_block(m, n, r));
    TSR_TRY(check_dtype(g_dtype));
    TSR_TRY(check_prec(precision));
    if (!G || !U || !V || !C || !ws) return TSR_INVALID_ARG;
    if (ldg < n) return TSR_BAD_SHAPE;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_project_workspace_bytes(m, n, r)) return TSR_WORKSPACE_TOO_SMALL;
    std::vector<BlockView> v;
    one_block_view(v, G, g_dtype, m, n, r, ldg, nullptr, n, (float*)U, (float*)V, C, nullptr);
    Arena ar(ws);
    ProjectProgram pg;
    build_project(pg, v, 1, precision, ar);
    Ctx cx{(hipStream_t)stream, nullptr};
    return run_project(pg, false, alpha, accumulate ? 1.0f : 0.0f, cx);
}

// ---------------------------------------------------------------- project, nothing allocated
}  // extern "C"

// Scratch of tsr_project_core_static: a fixed array in the code object, so every device that
// loads the library holds its own copy at its own address until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels get the looked-up address.
static __device__ __align__(256) unsigned char scratch[TSR_PROJECT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
    int dev = -1;
    TSR_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return TSR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        TSR_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr) return TSR_INVALID_ARG;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TSR_OK;
}
}  // namespace

extern "C" {

int tsr_project_core_static(const void* G, int g_dtype, int m, int n, long long ldg, const float* U, const float* V,
                            int r, float alpha, int accumulate, float* C, int precision, void* stream) {
    TSR_TRY(check_block(m, n, r));
    TSR_TRY(check_dtype(g_dtype));
    TSR_TRY(check_prec(precision));
    if (!G || !U || !V || !C) return TSR_INVALID_ARG;
    if (ldg < n) return TSR_BAD_SHAPE;
    if (tsr_project_workspace_bytes(m, n, r) > (size_t)TSR_PROJECT_STATIC_SCRATCH_BYTES) return TSR_STATIC_SCRATCH_TOO_SMALL;
    void* ws = nullptr;
    TSR_TRY(static_scratch(&ws));
    // every byte of the scratch that the kernels read (P = G V and the k-split partial cores) is
    // written earlier in the same call: nothing has to start at zero, so nothing is cleared
    std::vector<BlockView> v;
    one_block_view(v, G, g_dtype, m, n, r, ldg, nullptr, n, (float*)U, (float*)V, C, nullptr);
    Arena ar(ws);
    ProjectProgram pg;
    build_project(pg, v, 1, precision, ar);
    Ctx cx{(hipStream_t)stream, nullptr};
    return run_project(pg, false, alpha, accumulate ? 1.0f : 0.0f, cx);
}

// ---------------------------------------------------------------- average
int tsr_core_average(const float* Cs, int K, int r, float* Cbar, void* stream) {
    if (!Cs || !Cbar) return TSR_INVALID_ARG;
    if (K <= 0 || r <= 0) return TSR_BAD_SHAPE;
    TSR_HIP(launch_average(Cs, K, (long long)r * r, Cbar, (hipStream_t)stream));
    return TSR_OK;
}

// ---------------------------------------------------------------- calibration stream
int tsr_stream_scale(float* dst, const float* src, long long count, float scale, void* stream) {
    if (!dst || !src) return TSR_INVALID_ARG;
    if (count <= 0 || (count % 4) != 0) return TSR_BAD_SHAPE;
    if (((uintptr_t)dst % 16) || ((uintptr_t)src % 16)) return TSR_INVALID_ARG;
    TSR_HIP(launch_stream(dst, src, count, scale, (hipStream_t)stream));
    return TSR_OK;
}

// ---------------------------------------------------------------- Adam / SGD on the core
static int adam_scalars(AdamScalars& s, int t, float beta1, float beta2, float eps) {
    if (t < 1) return TSR_INVALID_ARG;
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) || !(eps >= 0.0f)) return TSR_INVALID_ARG;
    s.beta1 = beta1; s.beta2 = beta2; s.eps = eps;
    s.inv_c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)t)));
    s.inv_c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)t)));
    return TSR_OK;
}

int tsr_adam_core(const float* C, float* M, float* Vm, float* D, long long count, int t, float beta1, float beta2,
                  float eps, void* stream) {
    if (!C || !M || !Vm || !D) return TSR_INVALID_ARG;
    if (count <= 0) return TSR_BAD_SHAPE;
    AdamScalars s;
    TSR_TRY(adam_scalars(s, t, beta1, beta2, eps));
    CoreBlock b{C, M, Vm, D, count};
    TSR_HIP(launch_adam(nullptr, &b, 1, count, s, (hipStream_t)stream));
    return TSR_OK;
}

int tsr_sgd_core(const float* C, float* M, float* D, long long count, float beta, void* stream) {
    if (!C || !M || !D) return TSR_INVALID_ARG;
    if (count <= 0) return TSR_BAD_SHAPE;
    if (!(beta >= 0.0f && beta < 1.0f)) return TSR_INVALID_ARG;
    TSR_HIP(launch_sgd(C, M, D, count, beta, (hipStream_t)stream));
    return TSR_OK;
}

// ---------------------------------------------------------------- lift + apply
size_t tsr_backproject_workspace_bytes(int m, int n, int r) {
    if (check_block(m, n, r) != TSR_OK) return 0;
    std::vector<BlockView> v;
    one_block_view(v, nullptr, TSR_F32, m, n, r, n, nullptr, n, nullptr, nullptr, nullptr, nullptr);
    Arena ar(nullptr);
    LiftProgram lp;
    build_lift(lp, v, TSR_PREC_SPLIT, ar);
    return ar.used();
}

int tsr_backproject_apply(float* W, int m, int n, long long ldw, const float* U, const float* V, const float* D,
                          int r, float lr, float wd, float scale, int precision, void* ws, size_t ws_bytes,
                          void* stream) {
    TSR_TRY(check_block(m, n, r));
    TSR_TRY(check_prec(precision));
    if (!W || !U || !V || !D || !ws) return TSR_INVALID_ARG;
    if (ldw < n) return TSR_BAD_SHAPE;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_backproject_workspace_bytes(m, n, r)) return TSR_WORKSPACE_TOO_SMALL;
    std::vector<BlockView> v;
    one_block_view(v, nullptr, TSR_F32, m, n, r, n, W, ldw, (float*)U, (float*)V, nullptr, (float*)D);
    Arena ar(ws);
    LiftProgram lp;
    build_lift(lp, v, precision, ar);
    Ctx cx{(hipStream_t)stream, nullptr};
    return run_lift(lp, false, lr, wd, scale, cx);
}

// ---------------------------------------------------------------- refresh
size_t tsr_refresh_workspace_bytes(int m, int n, int r, int p) {
    if (check_refresh_shape(m, n, r, p) != TSR_OK) return 0;
    std::vector<BlockView> v;
    one_block_view(v, nullptr, TSR_F32, m, n, r, n, nullptr, n, nullptr, nullptr, nullptr, nullptr);
    Arena ar(nullptr);
    RefreshProgram rp;
    build_refresh(rp, v, nullptr, p, nullptr, ar);
    return ar.used();
}

int tsr_refresh_rsvd(const void* G, int g_dtype, int m, int n, long long ldg, const float* Omega, int r, int p,
                     int q, float* U, float* V, float* sigma, void* ws, size_t ws_bytes, void* stream) {
    TSR_TRY(check_refresh_shape(m, n, r, p));
    TSR_TRY(check_dtype(g_dtype));
    if (q < 0) return TSR_INVALID_ARG;
    if (!G || !Omega || !U || !V || !ws) return TSR_INVALID_ARG;
    if (ldg < n) return TSR_BAD_SHAPE;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_refresh_workspace_bytes(m, n, r, p)) return TSR_WORKSPACE_TOO_SMALL;
    std::vector<BlockView> v;
    one_block_view(v, G, g_dtype, m, n, r, ldg, nullptr, n, U, V, nullptr, nullptr);
    Arena ar(ws);
    RefreshProgram rp;
    const float* oms[1] = {Omega};
    float* sigs[1] = {sigma};
    build_refresh(rp, v, oms, p, sigs, ar);
    Ctx cx{(hipStream_t)stream, nullptr};
    return run_refresh(rp, false, q, cx);
}

size_t tsr_refresh_workers_workspace_bytes(int m, int n, int r, int p, int n_workers) {
    if (check_refresh_shape(m, n, r, p) != TSR_OK || n_workers <= 0) return 0;
    Arena ar(nullptr);
    const size_t k = (size_t)r + p;
    (void)ar.take<float>((size_t)n_workers * m * k);
    (void)ar.take<float>((size_t)n_workers * n * k);
    return ar.used() + tsr_refresh_workspace_bytes(m, n, r, p);
}

int tsr_refresh_rsvd_workers(const void* G, int g_dtype, int m, int n, long long ldg, long long g_stride,
                             int n_workers, const float* Omega, int r, int p, int q, float* U, float* V,
                             float* sigma, void* ws, size_t ws_bytes, void* stream) {
    TSR_TRY(check_refresh_shape(m, n, r, p));
    TSR_TRY(check_dtype(g_dtype));
    if (q < 0 || n_workers <= 0) return TSR_INVALID_ARG;
    if (!G || !Omega || !U || !V || !ws) return TSR_INVALID_ARG;
    if (ldg < n) return TSR_BAD_SHAPE;
    if (n_workers > 1 && g_stride < (long long)(m - 1) * ldg + n) return TSR_BAD_SHAPE;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_refresh_workers_workspace_bytes(m, n, r, p, n_workers)) return TSR_WORKSPACE_TOO_SMALL;
    const size_t k = (size_t)r + p;
    const size_t esz = (g_dtype == TSR_BF16) ? 2 : 4;
    Arena ar(ws);
    float* Qs = ar.take<float>((size_t)n_workers * m * k);     // the workers' Q_i, stacked
    float* Bs = ar.take<float>((size_t)n_workers * n * k);     // the workers' B_i^T, stacked
    const size_t mark = ar.used();
    Ctx cx{(hipStream_t)stream, nullptr};
    const float* oms[1] = {Omega};
    float* sigs[1] = {sigma};
    RefreshProgram rp;
    for (int w = 0; w < n_workers; ++w) {
        // the same buffers for every worker: only the gradient pointer differs
        std::vector<BlockView> v;
        one_block_view(v, (const char*)G + (size_t)w * g_stride * esz, g_dtype, m, n, r, ldg, nullptr, n, U, V, nullptr,
                       nullptr);
        Arena sub(ws);
        sub.off = mark;
        build_refresh(rp, v, oms, p, sigs, sub);
        TSR_TRY(run_refresh_front(rp, false, q, cx));
        const RefreshBlock& b = rp.blocks[0];
        TSR_HIP(hipMemcpyAsync(Qs + (size_t)w * m * k, b.Yalt, (size_t)m * k * sizeof(float), hipMemcpyDeviceToDevice, cx.s));
        TSR_HIP(hipMemcpyAsync(Bs + (size_t)w * n * k, b.Z, (size_t)n * k * sizeof(float), hipMemcpyDeviceToDevice, cx.s));
    }
    const RefreshBlock& b = rp.blocks[0];
    TSR_HIP(launch_average(Qs, n_workers, (long long)m * (long long)k, b.Yalt, cx.s));   // Qbar
    TSR_HIP(launch_average(Bs, n_workers, (long long)n * (long long)k, b.Z, cx.s));      // Bbar^T
    return run_refresh_back(rp, false, cx);
}

// ---------------------------------------------------------------- comparison paths of the ablations
// One-sided projection and lift on the grouped GEMM family, exact-SVD refresh on the back end of
// the randomized one (no sketch: the orthonormal basis of the short side is the identity).
}  // extern "C"

namespace {
struct OneSidedProgram { GemmStage proj[2], lift; };

// Ct (n x r) = alpha G^T U (+ Ct): the r x n one-sided object, stored transposed
void build_one_sided_project(OneSidedProgram& op, const void* G, int g_dtype, int m, int n, long long ldg, const float* U,
                             int r, float* Ct, int prec, Arena& ar) {
    std::vector<LogicalGemm> g{LogicalGemm{G, U, ldg, r, n, r, m, Ct, r}};
    const int pv = (prec == TSR_PREC_BF16) ? 1 : 2;
    build_stage(op.proj[g_dtype], variant(1, 1, g_dtype, pv, pv), g, ar);
}

// W = beta W + alpha U Dt^T with Dt (n x r) the transposed one-sided update
void build_one_sided_lift(OneSidedProgram& op, float* W, int m, int n, long long ldw, const float* U, const float* Dt,
                          int r, int prec, Arena& ar) {
    std::vector<LogicalGemm> g{LogicalGemm{U, Dt, r, r, m, n, r, W, ldw}};
    const int pv = (prec == TSR_PREC_BF16) ? 1 : 2;
    build_stage(op.lift, variant(0, 0, 0, pv, pv), g, ar, /*want_tiles=*/1);
}
}  // namespace

extern "C" {

size_t tsr_one_sided_workspace_bytes(int m, int n, int r) {
    if (m <= 0 || n <= 0 || r <= 0 || r > m) return 0;
    Arena ar(nullptr);
    OneSidedProgram op;
    build_one_sided_project(op, nullptr, TSR_F32, m, n, n, nullptr, r, nullptr, TSR_PREC_SPLIT, ar);
    build_one_sided_lift(op, nullptr, m, n, n, nullptr, nullptr, r, TSR_PREC_SPLIT, ar);
    return ar.used();
}

int tsr_project_one_sided(const void* G, int g_dtype, int m, int n, long long ldg, const float* U, int r, float alpha,
                          int accumulate, float* Ct, int precision, void* ws, size_t ws_bytes, void* stream) {
    if (m <= 0 || n <= 0 || r <= 0 || r > m) return TSR_BAD_SHAPE;
    TSR_TRY(check_dtype(g_dtype));
    TSR_TRY(check_prec(precision));
    if (!G || !U || !Ct || !ws) return TSR_INVALID_ARG;
    if (ldg < n) return TSR_BAD_SHAPE;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_one_sided_workspace_bytes(m, n, r)) return TSR_WORKSPACE_TOO_SMALL;
    Arena ar(ws);
    OneSidedProgram op;
    build_one_sided_project(op, G, g_dtype, m, n, ldg, U, r, Ct, precision, ar);
    Ctx cx{(hipStream_t)stream, nullptr};
    return run_stage(op.proj[g_dtype], false, alpha, accumulate ? 1.0f : 0.0f, cx, TSR_PROF_GV);
}

int tsr_backproject_one_sided(float* W, int m, int n, long long ldw, const float* U, const float* Dt, int r, float lr,
                              float wd, float scale, int precision, void* ws, size_t ws_bytes, void* stream) {
    if (m <= 0 || n <= 0 || r <= 0 || r > m) return TSR_BAD_SHAPE;
    TSR_TRY(check_prec(precision));
    if (!W || !U || !Dt || !ws) return TSR_INVALID_ARG;
    if (ldw < n) return TSR_BAD_SHAPE;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_one_sided_workspace_bytes(m, n, r)) return TSR_WORKSPACE_TOO_SMALL;
    Arena ar(ws);
    OneSidedProgram op;
    build_one_sided_lift(op, W, m, n, ldw, U, Dt, r, precision, ar);
    Ctx cx{(hipStream_t)stream, nullptr};
    return run_stage(op.lift, false, -lr * scale, 1.0f - lr * wd, cx, TSR_PROF_TVT);
}

// Exact SVD through the refresh back end: with s = min(m, n) the short side's basis is the s x s
// identity and the "reduced matrix" is the gradient itself, held as a tall (long side x s) fp32
// matrix T (G^T if m <= n, else G); then T = Q_T R, SVD of R, short-side vectors = X_r and
// long-side vectors = Q_T Gacc_r^T.  The short side plays the role of U's side in the block.
static int exact_svd_view(std::vector<BlockView>& v, int m, int n, int r, float* U, float* V) {
    const bool wide = (m <= n);            // short side = rows
    one_block_view(v, nullptr, TSR_F32, wide ? m : n, wide ? n : m, r, wide ? n : m, nullptr, 1, wide ? U : V, wide ? V : U,
                   nullptr, nullptr);
    return wide ? 1 : 0;
}

size_t tsr_refresh_exact_workspace_bytes(int m, int n, int r) {
    const int s = std::min(m, n);
    if (check_refresh_shape(m, n, r, s - r) != TSR_OK) return 0;
    std::vector<BlockView> v;
    exact_svd_view(v, m, n, r, nullptr, nullptr);
    Arena ar(nullptr);
    RefreshProgram rp;
    build_refresh(rp, v, nullptr, s - r, nullptr, ar);
    return ar.used();
}

int tsr_refresh_exact_svd(const void* G, int g_dtype, int m, int n, long long ldg, int r, float* U, float* V,
                          float* sigma, void* ws, size_t ws_bytes, void* stream) {
    TSR_TRY(check_block(m, n, r));
    const int s = std::min(m, n);
    TSR_TRY(check_refresh_shape(m, n, r, s - r));       // min(m, n) <= 1024: the small-SVD kernels' limit
    TSR_TRY(check_dtype(g_dtype));
    if (!G || !U || !V || !ws) return TSR_INVALID_ARG;
    if (ldg < n) return TSR_BAD_SHAPE;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_refresh_exact_workspace_bytes(m, n, r)) return TSR_WORKSPACE_TOO_SMALL;
    std::vector<BlockView> v;
    const int transpose = exact_svd_view(v, m, n, r, U, V);
    Arena ar(ws);
    RefreshProgram rp;
    float* sigs[1] = {sigma};
    build_refresh(rp, v, nullptr, s - r, sigs, ar);
    const RefreshBlock& b = rp.blocks[0];
    Ctx cx{(hipStream_t)stream, nullptr};
    TSR_HIP(launch_identity(b.Yalt, s, cx.s));                                          // Q = I (s x s)
    TSR_HIP(launch_tall_copy(G, g_dtype == TSR_BF16, ldg, m, n, transpose, b.Z, cx.s)); // B^T, tall
    return run_refresh_back(rp, false, cx);
}

// ---------------------------------------------------------------- moment re-alignment
}  // extern "C"

namespace {
struct RealignProgram { GemmStage a, b, am, out; };
void build_realign(RealignProgram& rp, const float* U_old, const float* V_old, const float* U_new, const float* V_new,
                   int m, int n, int r, float* M, Arena& ar) {
    float* A = ar.take<float>((size_t)r * r);       // U_new^T U_old
    float* B = ar.take<float>((size_t)r * r);       // V_old^T V_new
    float* AM = ar.take<float>((size_t)r * r);
    std::vector<LogicalGemm> ga{LogicalGemm{U_new, U_old, r, r, r, r, m, A, r}};
    std::vector<LogicalGemm> gb{LogicalGemm{V_old, V_new, r, r, r, r, n, B, r}};
    std::vector<LogicalGemm> gam{LogicalGemm{A, M, r, r, r, r, r, AM, r}};
    std::vector<LogicalGemm> gout{LogicalGemm{AM, B, r, r, r, r, r, M, r}};
    build_stage(rp.a, variant(1, 1, 0, 3, 3), ga, ar);
    build_stage(rp.b, variant(1, 1, 0, 3, 3), gb, ar);
    build_stage(rp.am, variant(0, 1, 0, 3, 3), gam, ar, 1);
    build_stage(rp.out, variant(0, 1, 0, 3, 3), gout, ar, 1);
}
}  // namespace

extern "C" {

size_t tsr_realign_workspace_bytes(int m, int n, int r) {
    if (check_block(m, n, r) != TSR_OK) return 0;
    Arena ar(nullptr);
    RealignProgram rp;
    build_realign(rp, nullptr, nullptr, nullptr, nullptr, m, n, r, nullptr, ar);
    return ar.used();
}

int tsr_realign_moment(const float* U_old, const float* V_old, const float* U_new, const float* V_new, int m, int n,
                       int r, float* M, void* ws, size_t ws_bytes, void* stream) {
    TSR_TRY(check_block(m, n, r));
    if (!U_old || !V_old || !U_new || !V_new || !M || !ws) return TSR_INVALID_ARG;
    if (!aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_realign_workspace_bytes(m, n, r)) return TSR_WORKSPACE_TOO_SMALL;
    Arena ar(ws);
    RealignProgram rp;
    build_realign(rp, U_old, V_old, U_new, V_new, m, n, r, M, ar);
    Ctx cx{(hipStream_t)stream, nullptr};
    TSR_TRY(run_stage(rp.a, false, 1.0f, 0.0f, cx, TSR_PROF_BASIS_GEMM));
    TSR_TRY(run_stage(rp.b, false, 1.0f, 0.0f, cx, TSR_PROF_BASIS_GEMM));
    TSR_TRY(run_stage(rp.am, false, 1.0f, 0.0f, cx, TSR_PROF_BASIS_GEMM));
    return run_stage(rp.out, false, 1.0f, 0.0f, cx, TSR_PROF_BASIS_GEMM);
}

// ---------------------------------------------------------------- plan
static int check_descs(const tsr_matrix_desc* descs, int count, int n_workers, int with_refresh, int p,
                       bool need_ptrs) {
    if (!descs || count <= 0 || n_workers <= 0) return TSR_INVALID_ARG;
    for (int i = 0; i < count; ++i) {
        const tsr_matrix_desc& d = descs[i];
        TSR_TRY(check_block(d.m, d.n, d.r));
        TSR_TRY(check_dtype(d.g_dtype));
        if (d.ldg < d.n || d.ldw < d.n) return TSR_BAD_SHAPE;
        if (n_workers > 1 && d.g_stride < (long long)(d.m - 1) * d.ldg + d.n) return TSR_BAD_SHAPE;
        if (with_refresh) TSR_TRY(check_refresh_shape(d.m, d.n, d.r, p));
        if (need_ptrs && (!d.G || !d.W || !d.U || !d.V || !d.M || !d.Vm || !d.C || !d.D)) return TSR_INVALID_ARG;
    }
    return TSR_OK;
}

static void views_from_descs(std::vector<BlockView>& v, const tsr_matrix_desc* descs, int count) {
    v.resize(count);
    for (int i = 0; i < count; ++i) {
        const tsr_matrix_desc& d = descs[i];
        BlockView b{};
        b.G = d.G; b.g_dtype = d.g_dtype; b.m = d.m; b.n = d.n; b.r = d.r; b.ldg = d.ldg; b.g_stride = d.g_stride;
        b.W = d.W; b.ldw = d.ldw; b.U = d.U; b.V = d.V; b.M = d.M; b.Vm = d.Vm; b.C = d.C; b.D = d.D;
        v[i] = b;
    }
}

// Builds every program of the plan into `ar`; with plan == nullptr only measures.
static void build_plan(tsr_plan& pl, Arena& ar) {
    pl.use_fast = (pl.precision == TSR_PREC_BF16) && !pl.force_generic && fast_step_eligible(pl.blocks, pl.n_workers);
    if (pl.use_fast) {
        build_fast_step(pl.fast, pl.blocks, pl.n_workers, ar);
    } else {
        build_project(pl.project, pl.blocks, pl.n_workers, pl.precision, ar);
        build_lift(pl.lift, pl.blocks, pl.precision, ar);
    }
    pl.cores.clear();
    pl.max_core = 0;
    for (const BlockView& b : pl.blocks) {
        const long long cnt = (long long)b.r * b.r;
        pl.cores.push_back(CoreBlock{b.C, b.M, b.Vm, b.D, cnt});
        pl.max_core = std::max(pl.max_core, cnt);
    }
    pl.groups.clear(); pl.group_blocks.clear();
    if (pl.with_refresh) {
        build_refresh(pl.refresh, pl.blocks, nullptr, pl.p, nullptr, ar, /*allow_nt=*/!pl.force_generic);
        const int ng = refresh_group_count((int)pl.blocks.size());
        if (ng > 1) {
            // heaviest blocks first onto the lightest group
            std::vector<int> order(pl.blocks.size());
            for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
            std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
                return (long long)pl.blocks[a].m * pl.blocks[a].n > (long long)pl.blocks[b].m * pl.blocks[b].n;
            });
            pl.group_blocks.assign(ng, {});
            std::vector<long long> load(ng, 0);
            for (int bi : order) {
                int best = 0;
                for (int g = 1; g < ng; ++g) if (load[g] < load[best]) best = g;
                pl.group_blocks[best].push_back(bi);
                load[best] += (long long)pl.blocks[bi].m * pl.blocks[bi].n;
            }
            pl.groups.resize(ng);
            for (int g = 0; g < ng; ++g) {
                std::sort(pl.group_blocks[g].begin(), pl.group_blocks[g].end());
                pl.groups[g].blocks.clear();
                for (int bi : pl.group_blocks[g]) pl.groups[g].blocks.push_back(pl.refresh.blocks[bi]);
                build_refresh_stages(pl.groups[g], nullptr, ar);
            }
        }
    }
    // device tables
    Uploader& up = pl.up;
    pl.d_cores = up.put(pl.cores, ar);
    if (pl.use_fast) {
        upload_fast_step(pl.fast, ar, up);
    } else {
        for (int d = 0; d < 2; ++d) upload_stage(pl.project.gv[d], ar, up);
        upload_stage(pl.project.utp, ar, up);
        upload_stage(pl.lift.ud, ar, up);
        upload_stage(pl.lift.tvt, ar, up);
    }
    if (pl.with_refresh) {
        upload_refresh(pl.refresh, ar, up);
        for (RefreshProgram& g : pl.groups) upload_refresh(g, ar, up);
    }
}

size_t tsr_plan_workspace_bytes(const tsr_matrix_desc* descs, int count, int n_workers, int precision,
                                int with_refresh, int p) {
    if (check_descs(descs, count, n_workers, with_refresh, p, false) != TSR_OK) return 0;
    if (check_prec(precision) != TSR_OK) return 0;
    tsr_plan pl;
    views_from_descs(pl.blocks, descs, count);
    pl.n_workers = n_workers; pl.precision = precision; pl.with_refresh = with_refresh != 0; pl.p = p;
    Arena ar(nullptr);
    build_plan(pl, ar);
    size_t need = ar.used();
    if (pl.use_fast) {
        // the gradient pointers given at creation may turn out unaligned: size for either path
        tsr_plan generic;
        generic.blocks = pl.blocks;
        generic.n_workers = n_workers; generic.precision = precision; generic.with_refresh = with_refresh != 0;
        generic.p = p; generic.force_generic = true;
        Arena ar2(nullptr);
        build_plan(generic, ar2);
        need = std::max(need, ar2.used());
    }
    return need;
}

int tsr_plan_create(const tsr_matrix_desc* descs, int count, int n_workers, int precision, int with_refresh, int p,
                    void* ws, size_t ws_bytes, void* stream, tsr_plan** plan_out) {
    if (!plan_out) return TSR_INVALID_ARG;
    *plan_out = nullptr;
    TSR_TRY(check_descs(descs, count, n_workers, with_refresh, p, true));
    TSR_TRY(check_prec(precision));
    if (!ws || !aligned256(ws)) return TSR_INVALID_ARG;
    if (ws_bytes < tsr_plan_workspace_bytes(descs, count, n_workers, precision, with_refresh, p))
        return TSR_WORKSPACE_TOO_SMALL;
    tsr_plan* pl = new (std::nothrow) tsr_plan;
    if (!pl) return TSR_INVALID_ARG;
    views_from_descs(pl->blocks, descs, count);
    pl->n_workers = n_workers; pl->precision = precision; pl->with_refresh = with_refresh != 0; pl->p = p;
    pl->ws = (char*)ws;
    Arena ar(ws);
    build_plan(*pl, ar);
    if (!pl->up.host.empty()) {
        hipError_t e = hipMemcpyAsync((char*)ws + pl->up.first, pl->up.host.data(), pl->up.host.size(),
                                      hipMemcpyHostToDevice, (hipStream_t)stream);
        if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
        if (e != hipSuccess) { delete pl; return hip_fail(e); }
    }
    if (pl->groups.size() > 1) {
        // side streams at the default priority; without them the refresh runs as one program
        bool ok = hipEventCreateWithFlags(&pl->fork, hipEventDisableTiming) == hipSuccess;
        for (size_t g = 1; ok && g < pl->groups.size(); ++g) {
            hipStream_t sg = nullptr; hipEvent_t ev = nullptr;
            ok = hipStreamCreateWithFlags(&sg, hipStreamNonBlocking) == hipSuccess;
            if (ok) pl->side.push_back(sg);
            ok = ok && hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess;
            if (ev) pl->joined.push_back(ev);
        }
        if (!ok) {
            // no side streams to be had: the refresh then runs as one program on the caller's stream
            (void)hipGetLastError();
            for (hipStream_t sg : pl->side) (void)hipStreamDestroy(sg);
            for (hipEvent_t ev : pl->joined) (void)hipEventDestroy(ev);
            pl->side.clear(); pl->joined.clear();
        }
    }
    *plan_out = pl;
    return TSR_OK;
}

void tsr_plan_destroy(tsr_plan* plan) { delete plan; }

int tsr_step_batched(tsr_plan* plan, int t, const tsr_hyper* h, void* stream) {
    if (!plan || !h) return TSR_INVALID_ARG;
    AdamScalars s;
    TSR_TRY(adam_scalars(s, t, h->beta1, h->beta2, h->eps));
    Ctx cx{(hipStream_t)stream, &plan->prof};
    if (plan->use_fast) return run_fast_step(plan->fast, plan->n_workers, s, h->lr, h->wd, h->scale, cx);
    TSR_TRY(run_project(plan->project, true, 1.0f / (float)plan->n_workers, 0.0f, cx));
    {
        Timed timed(cx, TSR_PROF_ADAM);
        TSR_HIP(launch_adam(plan->d_cores, nullptr, (int)plan->cores.size(), plan->max_core, s, cx.s));
    }
    return run_lift(plan->lift, true, h->lr, h->wd, h->scale, cx);
}

// Points the sketch stage of `rp` at this call's Omegas (om[i] belongs to rp.blocks[i]) and
// refreshes the device copy of those tables on `st`.
static int patch_omegas(RefreshProgram& rp, const std::vector<const float*>& om, hipStream_t st) {
    size_t cursor[2] = {0, 0}, nt_cursor = 0;
    for (size_t i = 0; i < rp.blocks.size(); ++i) {
        const int d = rp.blocks[i].g_dtype;
        if (rp.blocks[i].nt) rp.nt.s_om[nt_cursor++].X = om[i];
        else rp.sketch[d].probs[cursor[d]++].B = om[i];
    }
    for (int d = 0; d < 2; ++d) {
        GemmStage& sgm = rp.sketch[d];
        if (sgm.empty()) continue;
        TSR_HIP(hipMemcpyAsync((void*)sgm.d_probs, sgm.probs.data(), sgm.probs.size() * sizeof(GemmProblem),
                               hipMemcpyHostToDevice, st));
    }
    if (!rp.nt.empty())
        TSR_HIP(hipMemcpyAsync((void*)rp.nt.d_om, rp.nt.s_om.data(), rp.nt.s_om.size() * sizeof(SplitBlock),
                               hipMemcpyHostToDevice, st));
    return TSR_OK;
}

int tsr_refresh_batched(tsr_plan* plan, const float* const* Omegas, int q, void* stream) {
    if (!plan || !Omegas || q < 0) return TSR_INVALID_ARG;
    if (!plan->with_refresh) return TSR_INVALID_ARG;
    RefreshProgram& rp = plan->refresh;
    hipStream_t st = (hipStream_t)stream;
    for (size_t i = 0; i < rp.blocks.size(); ++i) if (!Omegas[i]) return TSR_INVALID_ARG;
    // with stage timing on, or with a single group, the whole refresh runs as one program
    const bool side_by_side = plan->groups.size() > 1 && !plan->prof.on && plan->side.size() + 1 == plan->groups.size();
    std::vector<const float*> om;
    if (side_by_side) {
        for (size_t g = 0; g < plan->groups.size(); ++g) {
            om.clear();
            for (int bi : plan->group_blocks[g]) om.push_back(Omegas[bi]);
            TSR_TRY(patch_omegas(plan->groups[g], om, st));
        }
    } else {
        om.assign(Omegas, Omegas + rp.blocks.size());
        TSR_TRY(patch_omegas(rp, om, st));
    }
    TSR_HIP(hipStreamSynchronize(st));
    plan->fast.bases_dirty = true;
    if (!side_by_side) {
        Ctx cx{st, &plan->prof};
        return run_refresh(rp, true, q, cx);
    }
    // fork: the side streams start after everything queued on the caller's stream so far
    TSR_HIP(hipEventRecord(plan->fork, st));
    // From here on an error does not return early: whatever was queued on a side stream is still
    // joined to the caller's stream, so that the caller's later work never overtakes it.
    int rc = TSR_OK;
    auto note = [&](hipError_t e) { if (e != hipSuccess && rc == TSR_OK) rc = hip_fail(e); };
    std::vector<char> forked(plan->groups.size(), 0);
    for (size_t g = 1; g < plan->groups.size(); ++g) {
        hipStream_t sg = plan->side[g - 1];
        const hipError_t e = hipStreamWaitEvent(sg, plan->fork, 0);
        note(e);
        if (e != hipSuccess) continue;                       // nothing queued on this side stream
        forked[g] = 1;
        Ctx cg{sg, nullptr};
        const int r = run_refresh(plan->groups[g], true, q, cg);
        if (rc == TSR_OK) rc = r;
    }
    {
        Ctx c0{st, nullptr};
        const int r = run_refresh(plan->groups[0], true, q, c0);
        if (rc == TSR_OK) rc = r;
    }
    // join: the caller's stream continues when every group is done
    for (size_t g = 1; g < plan->groups.size(); ++g) {
        if (!forked[g]) continue;
        const hipError_t e = hipEventRecord(plan->joined[g - 1], plan->side[g - 1]);
        note(e);
        if (e == hipSuccess) note(hipStreamWaitEvent(st, plan->joined[g - 1], 0));
        else note(hipStreamSynchronize(plan->side[g - 1]));   // no event to wait on: drain the side stream here
    }
    return rc;
}

int tsr_plan_kernel_path(const tsr_plan* plan) { return plan ? (plan->use_fast ? 1 : 0) : -1; }

int tsr_plan_bases_changed(tsr_plan* plan) {
    if (!plan) return TSR_INVALID_ARG;
    plan->fast.bases_dirty = true;
    return TSR_OK;
}

int tsr_plan_profile_begin(tsr_plan* plan) {
    if (!plan) return TSR_INVALID_ARG;
    plan->prof.clear();
    plan->prof.on = true;
    return TSR_OK;
}

int tsr_plan_profile_end(tsr_plan* plan, void* stream, float* ms, int* launches) {
    if (!plan || !ms) return TSR_INVALID_ARG;
    plan->prof.on = false;
    for (int i = 0; i < TSR_PROF_KINDS; ++i) { ms[i] = 0.0f; if (launches) launches[i] = 0; }
    TSR_HIP(hipStreamSynchronize((hipStream_t)stream));
    for (const Prof::Span& sp : plan->prof.spans) {
        float t = 0.0f;
        TSR_HIP(hipEventElapsedTime(&t, sp.a, sp.b));
        ms[sp.kind] += t;
        if (launches) launches[sp.kind] += 1;
    }
    plan->prof.clear();
    return TSR_OK;
}

void tsr_plan_payload_bytes(const tsr_plan* plan, int bytes_per_dense_element, long long* core_bytes,
                            long long* dense_bytes) {
    long long c = 0, d = 0;
    if (plan) {
        for (const BlockView& b : plan->blocks) {
            c += 4LL * b.r * b.r;
            d += (long long)bytes_per_dense_element * b.m * b.n;
        }
    }
    if (core_bytes) *core_bytes = c;
    if (dense_bytes) *dense_bytes = d;
}

}  // extern "C"
