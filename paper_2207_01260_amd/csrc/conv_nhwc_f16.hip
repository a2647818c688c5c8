// Instantiations of the channels-last implicit-GEMM convolution kernel for _Float16 data.
#include "conv_nhwc_kernel.hpp"

namespace cprune {

void launch_conv_nhwc_f16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup) {
  launch_tile_nhwc<_Float16>(tile, grid, s, a, fixup);
}

}  // namespace cprune
