// Instantiations of the 32x32-block spatial-patch convolution kernel for _Float16 data.
#include "conv_patch32_kernel.hpp"

namespace cprune {

void launch_conv_patch32_f16(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
  launch_patch32<_Float16>(id, grid, s, a);
}

}  // namespace cprune
