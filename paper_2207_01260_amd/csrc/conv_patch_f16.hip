// Instantiations of the 3x3 spatial-patch convolution kernel for _Float16 data.
#include "conv_patch_kernel.hpp"

namespace cprune {

void launch_conv_patch_f16(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
  launch_patch<_Float16>(id, grid, s, a);
}

}  // namespace cprune
