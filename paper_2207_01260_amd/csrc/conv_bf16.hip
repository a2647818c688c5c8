// Instantiations of the implicit-GEMM convolution kernel for __bf16 data.
#include "conv_kernel.hpp"

namespace cprune {

void launch_conv_bf16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup) {
  launch_tile<__bf16>(tile, grid, s, a, fixup);
}

}  // namespace cprune
