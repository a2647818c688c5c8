// Instantiations of the channels-last implicit-GEMM convolution kernel for __bf16 data.
#include "conv_nhwc_kernel.hpp"

namespace cprune {

void launch_conv_nhwc_bf16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup) {
  launch_tile_nhwc<__bf16>(tile, grid, s, a, fixup);
}

}  // namespace cprune
