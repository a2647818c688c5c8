// Instantiations of the 32x32-block spatial-patch convolution kernel for __bf16 data.
#include "conv_patch32_kernel.hpp"

namespace cprune {

void launch_conv_patch32_bf16(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
  launch_patch32<__bf16>(id, grid, s, a);
}

}  // namespace cprune
