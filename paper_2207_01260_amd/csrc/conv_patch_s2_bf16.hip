// Instantiations of the stride-2 spatial-patch 3x3 kernel for __bf16 data.
#include "conv_patch_kernel.hpp"

namespace cprune {

void launch_conv_patch_s2_bf16(int id, dim3 grid, hipStream_t s, const PatchArgs& a) { launch_patch_s2<__bf16>(id, grid, s, a); }

}  // namespace cprune
