// Instantiations of the 3x3 spatial-patch convolution kernel for float data.
#include "conv_patch_kernel.hpp"

namespace cprune {

void launch_conv_patch_f32(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
  launch_patch<float>(id, grid, s, a);
}

}  // namespace cprune
