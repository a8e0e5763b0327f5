// The bf16 per-step path: every contraction of project / lift as a k-contiguous bf16 NT GEMM
// over bf16 shadows of the bases (internal interface).
#pragma once
#include <vector>

#include "gemm.h"
#include "host_util.h"
#include "lift.h"
#include "nt_gemm.h"
#include "small.h"

namespace tsr {

struct NtStageH {
    NtVariant var{};
    std::vector<NtProblem> probs;
    std::vector<NtTile> tiles;            // XCD-interleaved, idle entries have prob < 0; or grouped by list
    std::vector<NtRange> ranges;          // persistent launch: one list of tiles per workgroup
    const NtRange* d_ranges = nullptr;
    std::vector<ReduceProblem> reduces;   // empty when the GEMM writes its output directly
    int max_reduce_elems = 0;
    const NtProblem* d_probs = nullptr;
    const NtTile* d_tiles = nullptr;
    const ReduceProblem* d_reduces = nullptr;
    bool empty() const { return probs.empty(); }
};

// One GEMM of a stage, C = A B^T in the NT family's operand form.
struct NtLogical {
    const void* A; const void* B; void* out;
    long long lda, ldb, ldc;
    int M, N, K;
    int block;      // owning matrix block (tiles of one block stay on one XCD)
    int group;      // consecutive entries with the same group >= 0 are summed into `out`
    long long b_piece_stride = 0;   // NtVariant::b_pieces > 1: elements between the pieces of B
};

// Tile lists, k splits and partial buffers of one launch (want_tiles: split k while the launch has
// fewer tiles; persistent: one list of tiles per workgroup; group_m: see the definition), its device
// tables, and the launch itself (plus the fixed-order reduction of k-split partials).
// lower_only: symmetric outputs of which only the tiles on or below the diagonal are computed.
void build_nt_stage(NtStageH& st, const NtVariant& var, const std::vector<NtLogical>& gemms, int n_blocks, Arena& ar,
                    int want_tiles, bool persistent = false, int group_m = 0, bool lower_only = false);
void upload_nt_stage(NtStageH& st, Arena& ar, Uploader& up);
int run_nt_stage(const NtStageH& st, float alpha, float beta, Ctx& cx, int kind, const AdamScalars* adam = nullptr);

struct FastStep {
    std::vector<ShadowBlock> shadows;  const ShadowBlock* d_shadows = nullptr;
    int max_rows = 0, max_r = 0;
    NtStageH gv[2];      // P^T = V^T G^T   (index: dtype of G), blocks the projection kernel cannot take
    struct ProjGroup {   // bf16 gradients of one rank handled by the projection kernel
        int r = 0, panel_rows = 128, depth = 2;
        std::vector<ProjItem> items;  const ProjItem* d_items = nullptr;
    };
    std::vector<ProjGroup> projs;
    NtStageH utp;        // C = U^T P
    std::vector<AdamTBlock> adam;  const AdamTBlock* d_adam = nullptr;
    NtStageH ud;         // T = U D                      (blocks the fused kernel cannot take)
    NtStageH tvt;        // W = beta W + alpha T V^T
    struct LiftGroup {   // blocks of one rank handled by the fused lift kernel
        int r = 0;
        int mode = 0;        // kernel variant (panel height / prefetch), see lift.hip
        std::vector<LiftBlock> blocks;  const LiftBlock* d_blocks = nullptr;
        std::vector<LiftTile> tiles;    const LiftTile* d_tiles = nullptr;     // work items, grouped by list
        std::vector<LiftRange> ranges;  const LiftRange* d_ranges = nullptr;   // one list of items per workgroup
    };
    std::vector<LiftGroup> lifts;
    bool adam_fused = false;   // the U^T P launch also runs Adam on each core (no separate Adam kernel)
    bool bases_dirty = true;
};

bool fast_step_eligible(const std::vector<BlockView>& blocks, int n_workers);
void build_fast_step(FastStep& fs, const std::vector<BlockView>& blocks, int n_workers, Arena& ar);
void upload_fast_step(FastStep& fs, Arena& ar, Uploader& up);
int run_fast_step(FastStep& fs, int n_workers, const AdamScalars& s, float lr, float wd, float scale, Ctx& cx);

}  // namespace tsr
