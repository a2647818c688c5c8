// Instantiations of the implicit-GEMM convolution kernel for float data.
#include "conv_kernel.hpp"

namespace cprune {

void launch_conv_f32(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup) {
  launch_tile<float>(tile, grid, s, a, fixup);
}

}  // namespace cprune
