// Instantiations of the implicit-GEMM convolution kernel for _Float16 data.
#include "conv_kernel.hpp"

namespace cprune {

void launch_conv_f16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup) {
  launch_tile<_Float16>(tile, grid, s, a, fixup);
}

}  // namespace cprune
