// Fused lift-and-apply kernel of the bf16 step path (internal interface): see lift.hip.
#pragma once
#include <hip/hip_runtime.h>

namespace tsr {

struct LiftBlock {
    const void* Ub;      // m x r bf16, leading dimension ldr
    const void* DTb;     // r x r bf16 (D transposed), leading dimension ldr
    const void* Vb;      // n x r bf16, leading dimension ldr
    float* W;            // m x n fp32, leading dimension ldw
    long long ldr, ldw;
    int m, n, r;
};

struct LiftTile { int block, row0, ct0, nct; };   // rows row0..row0+panel-1, 128-column tiles ct0..ct0+nct-1; block < 0: idle

bool lift_supports_rank(int r);
int lift_panel_rows(int mode);
hipError_t launch_lift(const LiftBlock* blocks_dev, const LiftTile* tiles_dev, int n_tiles, int r, bool vec4, int mode,
                       float alpha, float beta, hipStream_t stream);

}  // namespace tsr
