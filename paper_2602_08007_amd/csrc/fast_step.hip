// Launch-sequence builder of the bf16 per-step path (see fast_step.h).
#include "fast_step.h"

#include <algorithm>
#include <cstdlib>
#include <map>
#include <numeric>

namespace tsr {

namespace {

inline int cdiv(int a, int b) { return (a + b - 1) / b; }
inline long long round8(long long x) { return (x + 7) / 8 * 8; }
constexpr int N_XCD = 8;

// Workgroups are dealt to the 8 XCDs round-robin by linear id, and each XCD has its own L2:
// give every block to one XCD (greedy by work) and interleave the per-XCD tile lists, so the
// tiles that re-read a block's operands hit the L2 that already holds them.
// Tuning knobs read from the environment at plan creation (integers; unset = the built-in,
// measured-best choice): TSR_TUNE_XCD=0 keeps the natural tile order, TSR_TUNE_LPT=0 the block
// order within an XCD, TSR_TUNE_GV_BAND / TVT_BAND the tile-row bands of those stages,
// TSR_TUNE_GV_PERSIST / UTP_PERSIST the persistent launch of a stage, TSR_TUNE_UTP_TILES the tile
// count U^T P is split towards, TSR_TUNE_PROJ=0 routes G V through the NT family instead of the
// projection kernel (TSR_TUNE_PROJ_DEPTH: its pipeline depth), TSR_TUNE_FUSED_LIFT=0 uses the
// two-GEMM lift, TSR_TUNE_LIFT_MODE / LIFT_SETUP / LIFT_CUS shape the fused lift kernel's items
// and work lists, TSR_TUNE_ADAM_FUSED=0 keeps Adam out of the U^T P epilogue.  Which tile shape a
// stage runs on is a rule of the rank, not a knob.
int tune_int(const char* name, int dflt, int lo, int hi) {
    const char* v = std::getenv(name);
    if (!v || !*v) return dflt;
    const int x = std::atoi(v);
    return (x >= lo && x <= hi) ? x : dflt;
}
int tune(const char* name, int dflt) { return tune_int(name, dflt, 0, NT_SHAPES - 1); }

template <typename TileT>
void interleave_xcd(std::vector<TileT>& tiles, const std::vector<int>& tile_block, const std::vector<long long>& tile_work,
                    int n_blocks, const TileT& idle) {
    if (tune("TSR_TUNE_XCD", 1) == 0) return;
    std::vector<long long> work(n_blocks, 0);
    for (size_t i = 0; i < tiles.size(); ++i) work[tile_block[i]] += tile_work[i];
    std::vector<int> order(n_blocks);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return work[a] > work[b]; });
    std::vector<int> xcd_of(n_blocks, 0);
    long long load[N_XCD] = {0};
    for (int b : order) {
        int best = 0;
        for (int x = 1; x < N_XCD; ++x) if (load[x] < load[best]) best = x;
        xcd_of[b] = best;
        load[best] += work[b];
    }
    // Within an XCD the tiles with the longest contraction go first (stable: the tiles of one block
    // keep their order and stay neighbours), so that the launch does not end on its longest tiles.
    std::vector<size_t> idx(tiles.size());
    std::iota(idx.begin(), idx.end(), (size_t)0);
    if (tune("TSR_TUNE_LPT", 1) != 0)
        std::stable_sort(idx.begin(), idx.end(), [&](size_t a, size_t b) { return tile_work[a] > tile_work[b]; });
    std::vector<TileT> lists[N_XCD];
    for (size_t i : idx) lists[xcd_of[tile_block[i]]].push_back(tiles[i]);
    size_t longest = 0;
    for (auto& l : lists) longest = std::max(longest, l.size());
    std::vector<TileT> out;
    out.reserve(longest * N_XCD);
    for (size_t s = 0; s < longest; ++s)
        for (int x = 0; x < N_XCD; ++x) out.push_back(s < lists[x].size() ? lists[x][s] : idle);
    tiles.swap(out);
}

// Persistent launch: the tiles of each XCD's blocks are dealt to that XCD's workgroups, heaviest
// first onto the lightest list, and each list keeps the natural tile order (tiles that share an
// operand stay neighbours).  List j of XCD x belongs to workgroup 8 j + x.
void persistent_lists(std::vector<NtTile>& tiles, std::vector<NtRange>& ranges, const std::vector<int>& tile_block,
                      const std::vector<long long>& tile_work, int n_blocks, int lists_per_xcd) {
    std::vector<long long> work(n_blocks, 0);
    for (size_t i = 0; i < tiles.size(); ++i) work[tile_block[i]] += tile_work[i];
    std::vector<int> order(n_blocks);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return work[a] > work[b]; });
    std::vector<int> xcd_of(n_blocks, 0);
    long long load[N_XCD] = {0};
    for (int b : order) {
        int best = 0;
        for (int x = 1; x < N_XCD; ++x) if (load[x] < load[best]) best = x;
        xcd_of[b] = best;
        load[best] += work[b];
    }
    std::vector<NtTile> out;
    out.reserve(tiles.size());
    ranges.assign((size_t)N_XCD * lists_per_xcd, NtRange{0, 0});
    for (int x = 0; x < N_XCD; ++x) {
        std::vector<int> mine;
        for (size_t i = 0; i < tiles.size(); ++i) if (xcd_of[tile_block[i]] == x) mine.push_back((int)i);
        std::vector<int> by_work = mine;
        std::stable_sort(by_work.begin(), by_work.end(), [&](int a, int b) { return tile_work[a] > tile_work[b]; });
        std::vector<long long> lw(lists_per_xcd, 0);
        std::vector<std::vector<int>> lists(lists_per_xcd);
        for (int i : by_work) {
            int best = 0;
            for (int j = 1; j < lists_per_xcd; ++j) if (lw[j] < lw[best]) best = j;
            lists[best].push_back(i);
            lw[best] += tile_work[i];
        }
        for (int j = 0; j < lists_per_xcd; ++j) {
            std::sort(lists[j].begin(), lists[j].end());
            NtRange& r = ranges[(size_t)N_XCD * j + x];
            r.begin = (int)out.size();
            for (int i : lists[j]) out.push_back(tiles[i]);
            r.end = (int)out.size();
        }
    }
    tiles.swap(out);
}

}  // namespace

// group_m: order of a problem's output tiles within one k split.  0: row of tiles after row of
// tiles.  g > 0: bands of g tile rows, and inside a band column after column (the g tiles of a
// column are neighbours).  The workgroups resident on an XCD at one time then cover a compact patch
// of the output: they share g row panels of A, which stay in that XCD's L2 for the whole band, and
// each column panel of B is fetched once per band instead of once per tile row.
void build_nt_stage(NtStageH& st, const NtVariant& var, const std::vector<NtLogical>& gemms, int n_blocks, Arena& ar,
                    int want_tiles, bool persistent, int group_m, bool lower_only) {
    st = NtStageH{};
    st.var = var;
    if (gemms.empty()) return;
    const int TM = nt_tile_m(var.shape), TN = nt_tile_n(var.shape);
    long long base_tiles = 0;
    bool shared = false;
    for (size_t i = 0; i < gemms.size(); ++i) {
        base_tiles += (long long)cdiv(gemms[i].M, TM) * cdiv(gemms[i].N, TN);
        if (i > 0 && gemms[i].group >= 0 && gemms[i].group == gemms[i - 1].group) shared = true;
    }
    const int want_split = (int)std::max<long long>(1, want_tiles / std::max<long long>(1, base_tiles));
    std::vector<int> ksplit(gemms.size()), kchunk(gemms.size());
    bool any_split = false;
    for (size_t i = 0; i < gemms.size(); ++i) {
        const int K = gemms[i].K;
        int s = std::min(want_split, std::max(1, K / 256));
        int chunk = cdiv(cdiv(K, s), 64) * 64;
        s = cdiv(K, chunk);
        ksplit[i] = s; kchunk[i] = chunk;
        if (s > 1) any_split = true;
    }
    const bool direct = !(any_split || shared);
    st.probs.resize(gemms.size());
    std::vector<int> tile_block;
    std::vector<long long> tile_work;
    size_t i = 0;
    while (i < gemms.size()) {
        size_t e = i + 1;
        while (e < gemms.size() && gemms[i].group >= 0 && gemms[e].group == gemms[i].group) ++e;
        const size_t mn = (size_t)gemms[i].M * gemms[i].N;
        float* part = nullptr;
        if (!direct) {
            int gs = 0;
            for (size_t j = i; j < e; ++j) gs += ksplit[j];
            part = ar.take<float>(mn * gs);
            ReduceProblem r{};
            r.part = part; r.out = (float*)gemms[i].out; r.stride = (long long)mn; r.ldc = gemms[i].ldc;
            r.M = gemms[i].M; r.N = gemms[i].N; r.splits = gs;
            st.reduces.push_back(r);
            st.max_reduce_elems = std::max(st.max_reduce_elems, (int)std::min<size_t>(mn, 1u << 30));
        }
        int prefix = 0;
        for (size_t j = i; j < e; ++j) {
            const NtLogical& g = gemms[j];
            NtProblem& p = st.probs[j];
            p.A = g.A; p.B = g.B; p.lda = g.lda; p.ldb = g.ldb; p.M = g.M; p.N = g.N; p.K = g.K;
            p.b_piece_stride = g.b_piece_stride;
            if (direct) {
                p.C = g.out; p.ldc = g.ldc; p.c_split_stride = 0; p.kchunk = std::max(64, cdiv(g.K, 64) * 64);
                ksplit[j] = 1;
            } else {
                p.C = part ? (void*)(part + mn * prefix) : nullptr;
                p.ldc = g.N; p.c_split_stride = (long long)mn; p.kchunk = kchunk[j];
                prefix += ksplit[j];
            }
            const int tmn = cdiv(g.M, TM), tnn = cdiv(g.N, TN);
            const int band = (group_m > 0) ? group_m : 1;
            for (int ks = 0; ks < ksplit[j]; ++ks)
                for (int tb = 0; tb < tmn; tb += band)
                    for (int t2 = 0; t2 < (group_m > 0 ? tnn : 1); ++t2)
                        for (int tm = tb; tm < std::min(tmn, tb + band); ++tm)
                            for (int t3 = 0; t3 < (group_m > 0 ? 1 : tnn); ++t3) {
                                if (lower_only && ((group_m > 0) ? t2 : t3) * TN > tm * TM + TM - 1) continue;
                                st.tiles.push_back(NtTile{(int)j, tm, (group_m > 0) ? t2 : t3, ks});
                                tile_block.push_back(g.block);
                                tile_work.push_back(std::min(p.kchunk, g.K) + 64);
                            }
        }
        i = e;
    }
    if (persistent)
        persistent_lists(st.tiles, st.ranges, tile_block, tile_work, n_blocks,
                         tune_int("TSR_TUNE_NT_CUS", 256, 8, 4096) / N_XCD * nt_wgs_per_cu(var.shape));
    else
        interleave_xcd(st.tiles, tile_block, tile_work, n_blocks, NtTile{-1, 0, 0, 0});
}

int run_nt_stage(const NtStageH& st, float alpha, float beta, Ctx& cx, int kind, const AdamScalars* adam) {
    if (st.empty()) return TSR_OK;
    Timed timed(cx, kind);
    NtLaunch L{};
    if (adam) L.adam = *adam;
    L.probs = st.d_probs; L.tiles = st.d_tiles; L.n_tiles = (int)st.tiles.size();
    if (!st.ranges.empty()) { L.ranges = st.d_ranges; L.n_tiles = (int)st.ranges.size(); }
    if (st.reduces.empty()) {
        L.alpha = alpha; L.beta = beta;
        TSR_HIP(launch_nt_gemm(L, st.var, cx.s));
    } else {
        L.alpha = 1.0f; L.beta = 0.0f;
        TSR_HIP(launch_nt_gemm(L, st.var, cx.s));
        TSR_HIP(launch_splitk_reduce(st.d_reduces, nullptr, (int)st.reduces.size(), st.max_reduce_elems, alpha, beta,
                                     cx.s));
    }
    return TSR_OK;
}

void upload_nt_stage(NtStageH& st, Arena& ar, Uploader& up) {
    if (st.empty()) return;
    st.d_probs = up.put(st.probs, ar);
    st.d_tiles = up.put(st.tiles, ar);
    if (!st.reduces.empty()) st.d_reduces = up.put(st.reduces, ar);
    if (!st.ranges.empty()) st.d_ranges = up.put(st.ranges, ar);
}

// The NT kernels fetch 16-byte chunks through 32-bit buffer offsets: every gradient needs a
// 16-byte aligned base, a row pitch (and worker stride) that is a multiple of 16 bytes and covers
// the column count rounded up to 8 elements, and tiles past the last row must still be
// addressable in 31 bits.
bool fast_step_eligible(const std::vector<BlockView>& blocks, int n_workers) {
    const long long lim = 1LL << 31;
    for (const BlockView& b : blocks) {
        const long long esz = (b.g_dtype == TSR_BF16) ? 2 : 4;
        // a 16-byte chunk that starts inside a row must end inside that row's pitch
        if (((uintptr_t)b.G) % 16 != 0 || (b.ldg * esz) % 16 != 0 || b.ldg < round8(b.n)) return false;
        if (n_workers > 1 && (b.g_stride * esz) % 16 != 0) return false;
        const long long big = std::max(b.m, b.n);
        if ((long long)(b.m + 256) * b.ldg * esz >= lim) return false;                  // G
        if ((big + 256) * round8(b.r) * 2 >= lim) return false;                          // U, V, T shadows
        if ((long long)(b.r + 256) * round8(big) * 2 >= lim) return false;               // U^T, V^T, P^T
        if ((long long)(b.m + 256) * b.ldw * 4 >= lim) return false;                     // W
    }
    return true;
}

void build_fast_step(FastStep& fs, const std::vector<BlockView>& blocks, int n_workers, Arena& ar) {
    fs.shadows.clear(); fs.adam.clear(); fs.lifts.clear(); fs.projs.clear();
    const bool use_proj_kernel = tune_int("TSR_TUNE_PROJ", 1, 0, 1) != 0;
    const int proj_rows = 128;
    // gradient tiles in flight per workgroup: 2 (measured best: two workgroups per compute unit) or 4 (one)
    const int proj_depth = tune_int("TSR_TUNE_PROJ_DEPTH", 2, 2, 4) == 4 ? 4 : 2;
    std::map<int, std::vector<int>> proj_block;
    std::map<int, std::vector<long long>> proj_work;
    fs.max_rows = 0; fs.max_r = 0;
    const bool fused_lift = tune_int("TSR_TUNE_FUSED_LIFT", 1, 0, 1) != 0;
    int r_all = 0;
    for (const BlockView& b : blocks) r_all = std::max(r_all, b.r);
    // ranks above 256: the wide-tile kernel for the two products with a bf16 output
    const int s1_shape = r_all > 256 ? NT_256x256_K32 : (r_all > 64 ? NT_128x128 : NT_64x256);
    const int ud_shape = r_all > 256 ? NT_256x256_K32 : NT_128x128, tvt_shape = NT_128x128;
    const int lift_cus = tune_int("TSR_TUNE_LIFT_CUS", 256, 8, 4096);       // compute units of the target
    const int lift_setup = tune_int("TSR_TUNE_LIFT_SETUP", 2, 0, 16);       // cost of an item's setup, in tiles
    const int lift_mode = tune_int("TSR_TUNE_LIFT_MODE", 2, 0, 2);
    std::vector<NtLogical> gv[2], utp, ud, tvt;
    const int nb = (int)blocks.size();
    int r_max = 0;
    for (int bi = 0; bi < nb; ++bi) {
        const BlockView& b = blocks[bi];
        const long long ldr = round8(b.r), ldm = round8(b.m), ldn = round8(b.n);
        typedef unsigned short bf;
        bf* Ub = ar.take<bf>((size_t)b.m * ldr);
        bf* UTb = ar.take<bf>((size_t)b.r * ldm);
        bf* Vb = ar.take<bf>((size_t)b.n * ldr);
        bf* VTb = ar.take<bf>((size_t)b.r * ldn);
        // The normalized update meets the basis of the shorter side: T = alpha U D (m x r) when m <= n, else
        // T = alpha V D^T (n x r), and the weight update is W <- beta W + T V^T resp. beta W + U T^T.
        const bool t_on_v = b.n < b.m && tune_int("TSR_TUNE_T_SHORT_SIDE", 1, 0, 1) != 0;
        bf* Tb = ar.take<bf>((size_t)(t_on_v ? b.n : b.m) * ldr);
        bf* DTb = ar.take<bf>((size_t)b.r * ldr);
        const bool fits32 = (long long)(b.m + 128) * b.ldw * 4 < (1LL << 31) && (long long)(std::max(b.m, b.n) + 128) * ldr * 2 < (1LL << 31);
        const bool use_lift = fused_lift && lift_supports_rank(b.r) && fits32;
        bf* Vf = use_lift ? ar.take<bf>((size_t)cdiv(b.n, 32) * 32 * b.r) : nullptr;
        const bool use_proj = use_proj_kernel && b.g_dtype == TSR_BF16 && proj_supports_rank(b.r) &&
                              (long long)b.r * (b.n + 16) * 2 < (1LL << 31);
        bf* VTf = use_proj ? ar.take<bf>((size_t)b.r * ((b.n + 15) / 16 * 16)) : nullptr;
        fs.shadows.push_back(ShadowBlock{b.U, Ub, UTb, nullptr, nullptr, b.m, b.r, ldr, ldm});
        fs.shadows.push_back(ShadowBlock{b.V, Vb, VTb, Vf, VTf, b.n, b.r, ldr, ldn});
        fs.max_rows = std::max(fs.max_rows, std::max(b.m, b.n));
        fs.max_r = std::max(fs.max_r, b.r);
        r_max = std::max(r_max, b.r);
        const int esz = (b.g_dtype == TSR_BF16) ? 2 : 4;
        for (int w = 0; w < n_workers; ++w) {
            bf* PT = ar.take<bf>((size_t)b.r * ldm);
            const char* Gw = b.G ? (const char*)b.G + (size_t)w * b.g_stride * esz : nullptr;
            if (use_proj) {
                FastStep::ProjGroup* pg = nullptr;
                for (auto& g : fs.projs) if (g.r == b.r) pg = &g;
                if (!pg) { fs.projs.emplace_back(); pg = &fs.projs.back(); pg->r = b.r; pg->panel_rows = proj_rows; pg->depth = proj_depth; }
                for (int row0 = 0; row0 < b.m; row0 += proj_rows) {
                    pg->items.push_back(ProjItem{Gw, VTf, PT, b.ldg, ldm, b.m, b.n, row0});
                    proj_block[b.r].push_back(bi);
                    proj_work[b.r].push_back(b.n + 64);
                }
            } else {
                gv[b.g_dtype].push_back(NtLogical{VTb, Gw, PT, ldn, b.ldg, ldm, b.r, b.m, b.n, bi, -1});
            }
            utp.push_back(NtLogical{UTb, PT, b.C, ldm, ldm, b.r, b.r, b.r, b.m, bi, bi});
        }
        bf* DTf = use_lift ? ar.take<bf>((size_t)b.r * b.r) : nullptr;
        bf* Db = (!use_lift && t_on_v) ? ar.take<bf>((size_t)b.r * ldr) : nullptr;
        fs.adam.push_back(AdamTBlock{b.C, b.M, b.Vm, b.D, DTb, DTf, b.r, ldr, Db});
        if (use_lift) {
            FastStep::LiftGroup* grp = nullptr;
            for (auto& g : fs.lifts) if (g.r == b.r) grp = &g;
            if (!grp) { fs.lifts.emplace_back(); grp = &fs.lifts.back(); grp->r = b.r; grp->mode = lift_mode; }
            const int bidx = (int)grp->blocks.size();
            grp->blocks.push_back(LiftBlock{Ub, DTf, Vf, b.W, ldr, b.ldw, b.m, b.n, b.r});
            // whole row panels for now; cut into per-workgroup lists below
            for (int row0 = 0; row0 < b.m; row0 += lift_panel_rows(lift_mode))
                grp->tiles.push_back(LiftTile{bidx, row0, 0, cdiv(b.n, 128)});
        } else {
            if (t_on_v) {
                ud.push_back(NtLogical{Vb, Db, Tb, ldr, ldr, ldr, b.n, b.r, b.r, bi, -1});
                tvt.push_back(NtLogical{Ub, Tb, b.W, ldr, ldr, b.ldw, b.m, b.n, b.r, bi, -1});
            } else {
                ud.push_back(NtLogical{Ub, DTb, Tb, ldr, ldr, ldr, b.m, b.r, b.r, bi, -1});
                tvt.push_back(NtLogical{Tb, Vb, b.W, ldr, ldr, b.ldw, b.m, b.n, b.r, bi, -1});
            }
        }
    }
    // Persistent launch: one list of work items per workgroup, all lists equally heavy (tiles
    // plus the setup cost of every item).  The panels are walked in block order and cut where a
    // list is full; list s goes to workgroup 8 (s mod L/8) + s / (L/8), so that the lists of
    // neighbouring panels (which share V) run on one XCD and share its L2.
    for (auto& g : fs.lifts) {
        const int n_lists = lift_cus * lift_wgs_per_cu(g.mode);
        std::vector<LiftTile> panels;
        panels.swap(g.tiles);
        long long total = 0;
        for (const LiftTile& p : panels) total += p.nct + lift_setup;
        // a cut adds one setup; `cap` is the smallest list weight that lets everything fit
        long long cap = std::max<long long>(cdiv(total, n_lists), lift_setup + 1);
        std::vector<std::vector<LiftTile>> lists;
        for (;; ++cap) {
            lists.assign(1, {});
            long long w = 0;
            for (const LiftTile& p : panels) {
                int c0 = 0;
                while (c0 < p.nct) {
                    if (cap - w < lift_setup + 1) { lists.emplace_back(); w = 0; }
                    const int take = (int)std::min<long long>(p.nct - c0, cap - w - lift_setup);
                    lists.back().push_back(LiftTile{p.block, p.row0, c0, take});
                    w += take + lift_setup;
                    c0 += take;
                }
            }
            if ((int)lists.size() <= n_lists) break;
        }
        g.ranges.assign(n_lists, LiftRange{0, 0});
        const int per_xcd = n_lists / 8;
        for (int s = 0; s < (int)lists.size(); ++s) {
            const int wg = (n_lists % 8 == 0) ? 8 * (s % per_xcd) + s / per_xcd : s;
            g.ranges[wg].begin = (int)g.tiles.size();
            g.tiles.insert(g.tiles.end(), lists[s].begin(), lists[s].end());
            g.ranges[wg].end = (int)g.tiles.size();
        }
    }
    for (auto& g : fs.projs) {
        // long contractions first: the hardware hands out panels in this order
        std::vector<int> idx(g.items.size());
        std::iota(idx.begin(), idx.end(), 0);
        std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return g.items[a].n > g.items[b].n; });
        std::vector<ProjItem> items; std::vector<int> blk; std::vector<long long> wk;
        for (int i : idx) { items.push_back(g.items[i]); blk.push_back(proj_block[g.r][i]); wk.push_back(proj_work[g.r][i]); }
        g.items.swap(items);
        ProjItem idle{};
        interleave_xcd(g.items, blk, wk, nb, idle);
    }
    // persistent launches pay off for the many short tiles of U^T P, not for the G V stage
    const bool gv_persist = tune_int("TSR_TUNE_GV_PERSIST", 0, 0, 1) != 0;
    const bool utp_persist = tune_int("TSR_TUNE_UTP_PERSIST", 1, 0, 1) != 0;
    // P^T = V^T G^T has r / 128 tile rows over every panel of G: all of them side by side, so that the
    // panel comes from memory once; W = beta W + T V^T in bands of four tile rows (measured: L2-to-fabric
    // reads 12.2 GB per launch without bands, 8.0 GB with bands of four or eight; 2.83 / 2.74 / 2.82 ms)
    const int gv_band = tune_int("TSR_TUNE_GV_BAND", 8, 0, 64), tvt_band = tune_int("TSR_TUNE_TVT_BAND", 4, 0, 64);
    // the shapes without a persistent form (wide tiles) always launch one tile per workgroup
    const bool gv_p = gv_persist && s1_shape != NT_256x256_K32;
    build_nt_stage(fs.gv[TSR_F32], NtVariant{(s1_shape == NT_256x256_K32) ? (int)NT_128x128 : s1_shape, 1, 1}, gv[TSR_F32], nb, ar, 1, gv_p, gv_band);
    build_nt_stage(fs.gv[TSR_BF16], NtVariant{s1_shape, 0, 1}, gv[TSR_BF16], nb, ar, 1, gv_p, gv_band);
    // cores up to 256 x 256 are cut into 64 x 64 tiles (enough of them to fill the chip without
    // splitting k); larger cores have enough 128 x 128 tiles
    // ... and above rank 256 the wide-tile kernel without a k split (four 256 x 256 tiles per core:
    // 0.31 ms against 0.37 ms for 128 x 128 tiles split towards 2048 on the 1B workload; with a
    // k split the wide tiles lose, 0.58 - 0.87 ms)
    const bool utp_wide = r_max >= 512 && tune_int("TSR_TUNE_UTP_WIDE", 1, 0, 1) != 0;
    build_nt_stage(fs.utp, NtVariant{utp_wide ? NT_256x256_K32 : (r_max >= 512 ? NT_128x128 : NT_64x64), 0, 0}, utp, nb, ar,
                   utp_wide ? 1 : tune_int("TSR_TUNE_UTP_TILES", 2048, 1, 65536), utp_persist && !utp_wide);
    build_nt_stage(fs.ud, NtVariant{ud_shape, 0, 1}, ud, nb, ar, 1);
    // At rank 512 the weight update runs on the wave-specialised kernel (persistent lists, one workgroup
    // per compute unit) when every problem fits it: K = 512 and a last column tile of at least four columns.
    bool tvt_ws = !tvt.empty() && tune_int("TSR_TUNE_TVT_WS", 1, 0, 1) != 0;
    for (const NtLogical& g : tvt) tvt_ws = tvt_ws && g.K == 512 && (g.N % 128 == 0 || g.N % 128 >= 4);
    build_nt_stage(fs.tvt, NtVariant{tvt_ws ? (int)NT_128x128_WS : tvt_shape, 0, 0}, tvt, nb, ar, 1, tvt_ws, tvt_band);
}

void upload_fast_step(FastStep& fs, Arena& ar, Uploader& up) {
    fs.d_shadows = up.put(fs.shadows, ar);
    fs.d_adam = up.put(fs.adam, ar);
    // Adam rides in the epilogue of U^T P when every core is written whole by that GEMM: one
    // worker, no k split, persistent launch, one problem per block in block order.  Only with
    // 64 x 64 tiles (cores up to 256 x 256): with the 128 x 128 tiles of larger cores the long
    // epilogue measured slower than the separate Adam kernel.
    fs.adam_fused = false;
    if (tune_int("TSR_TUNE_ADAM_FUSED", 1, 0, 1) != 0 && fs.utp.reduces.empty() && !fs.utp.ranges.empty() &&
        fs.utp.var.shape == NT_64x64 && fs.utp.probs.size() == fs.adam.size()) {
        bool ok = true;
        for (size_t j = 0; j < fs.adam.size(); ++j) {
            const NtProblem& p = fs.utp.probs[j];
            const AdamTBlock& a = fs.adam[j];
            ok = ok && p.C == (void*)a.C && p.M == a.r && p.N == a.r && p.ldc == a.r && (a.DTf == nullptr || a.r % 32 == 0);
        }
        if (ok) {
            for (size_t j = 0; j < fs.adam.size(); ++j) fs.utp.probs[j].adam = fs.d_adam + j;
            fs.utp.var.fused_adam = 1;
            fs.adam_fused = true;
        }
    }
    for (int d = 0; d < 2; ++d) upload_nt_stage(fs.gv[d], ar, up);
    for (auto& g : fs.projs) g.d_items = up.put(g.items, ar);
    upload_nt_stage(fs.utp, ar, up);
    upload_nt_stage(fs.ud, ar, up);
    upload_nt_stage(fs.tvt, ar, up);
    for (auto& g : fs.lifts) {
        g.d_blocks = up.put(g.blocks, ar);
        g.d_tiles = up.put(g.tiles, ar);
        g.d_ranges = up.put(g.ranges, ar);
    }
}

int run_fast_step(FastStep& fs, int n_workers, const AdamScalars& s, float lr, float wd, float scale, Ctx& cx) {
    if (fs.bases_dirty) {
        TSR_HIP(launch_shadows(fs.d_shadows, (int)fs.shadows.size(), fs.max_rows, fs.max_r, cx.s));
        fs.bases_dirty = false;
    }
    TSR_TRY(run_nt_stage(fs.gv[TSR_F32], 1.0f, 0.0f, cx, TSR_PROF_GV));
    TSR_TRY(run_nt_stage(fs.gv[TSR_BF16], 1.0f, 0.0f, cx, TSR_PROF_GV));
    for (const auto& g : fs.projs) {
        Timed timed(cx, TSR_PROF_GV);
        TSR_HIP(launch_proj(g.d_items, (int)g.items.size(), g.r, g.depth, cx.s));
    }
    TSR_TRY(run_nt_stage(fs.utp, 1.0f / (float)n_workers, 0.0f, cx, TSR_PROF_UTP, fs.adam_fused ? &s : nullptr));
    if (!fs.adam_fused) {
        Timed timed(cx, TSR_PROF_ADAM);
        TSR_HIP(launch_adam_t(fs.d_adam, (int)fs.adam.size(), fs.max_r, s, cx.s));
    }
    // T = alpha U D carries the step size; the weight kernels then add T V^T to beta W
    const float alpha = -lr * scale, beta = 1.0f - lr * wd;
    TSR_TRY(run_nt_stage(fs.ud, alpha, 0.0f, cx, TSR_PROF_UD));
    TSR_TRY(run_nt_stage(fs.tvt, 1.0f, beta, cx, TSR_PROF_TVT));
    for (const auto& g : fs.lifts) {
        Timed timed(cx, TSR_PROF_TVT);
        TSR_HIP(launch_lift(g.d_blocks, g.d_tiles, g.d_ranges, (int)g.ranges.size(), g.r, g.mode, alpha, beta, cx.s));
    }
    return TSR_OK;
}

}  // namespace tsr
