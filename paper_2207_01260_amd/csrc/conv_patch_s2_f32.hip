// Instantiations of the stride-2 spatial-patch 3x3 kernel for float data.
#include "conv_patch_kernel.hpp"

namespace cprune {

void launch_conv_patch_s2_f32(int id, dim3 grid, hipStream_t s, const PatchArgs& a) { launch_patch_s2<float>(id, grid, s, a); }

}  // namespace cprune
