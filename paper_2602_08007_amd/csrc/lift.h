// Fused lift-and-apply kernel of the bf16 step path (internal interface): see lift.hip.
#pragma once
#include <hip/hip_runtime.h>

namespace tsr {

struct LiftBlock {
    const void* Ub;      // m x r bf16, leading dimension ldr
    const void* DTf;     // D^T in fragment order (r/32 groups x r/16 steps x 1 KiB), see AdamTBlock::DTf
    const void* Vf;      // V in fragment order (ceil(n/32) groups x r/16 steps x 1 KiB), see ShadowBlock::XFb
    float* W;            // m x n fp32, leading dimension ldw
    long long ldr, ldw;
    int m, n, r;
};

struct LiftTile { int block, row0, ct0, nct; };   // work item: rows row0..row0+lift_panel_rows-1, 128-column tiles ct0..ct0+nct-1
struct LiftRange { int begin, end; };              // the items [begin, end) of one workgroup

bool lift_supports_rank(int r);
int lift_panel_rows(int mode);   // rows of an item
int lift_wgs_per_cu(int mode);
hipError_t launch_lift(const LiftBlock* blocks_dev, const LiftTile* tiles_dev, const LiftRange* ranges_dev, int n_wgs,
                       int r, int mode, float alpha, float beta, hipStream_t stream);

}  // namespace tsr
