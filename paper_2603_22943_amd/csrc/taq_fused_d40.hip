// Instantiations of the fused block kernel for (head dimension, heads) = (40, 8).
#include "taq_fused_kernel.h"

namespace taq {

hipError_t launch_fused_d40(const FusedTable& tab, const FusedDims& dm, int grid, int tok, bool core, hipStream_t st) {
    if (core) return launch_fused_cfg<40, 8, 2, 1, 32, true>(tab, dm, grid, st);
    return tok == 16 ? launch_fused_cfg<40, 8, 1, 1, 16>(tab, dm, grid, st) : launch_fused_cfg<40, 8, 2, 1>(tab, dm, grid, st);
}

}  // namespace taq
