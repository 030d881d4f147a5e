// Instantiations of the head-group variant of the fused block kernel for (head dimension, heads) = (160, 8): eight head groups of one head.
#include "taq_fused_kernel.h"

namespace taq {

hipError_t launch_fused_mid160(const FusedTable& tab, const FusedDims& dm, int grid, int tok, hipStream_t st) {
    return tok == 16 ? launch_fused_cfg<160, 1, 1, 8, 16>(tab, dm, grid, st) : launch_fused_cfg<160, 1, 1, 8>(tab, dm, grid, st);
}

}  // namespace taq
