// Instantiations of the head-group variant of the fused block kernel for (head dimension, heads) = (64, 20): ten head groups of two heads.
#include "taq_fused_kernel.h"

namespace taq {

hipError_t launch_fused_mid64(const FusedTable& tab, const FusedDims& dm, int grid, int tok, hipStream_t st) {
    return tok == 16 ? launch_fused_cfg<64, 2, 1, 10, 16>(tab, dm, grid, st) : launch_fused_cfg<64, 2, 1, 10>(tab, dm, grid, st);
}

}  // namespace taq
