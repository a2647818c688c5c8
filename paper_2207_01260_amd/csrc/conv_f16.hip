// Instantiations of the implicit-GEMM convolution kernel for _Float16 data.
#include "conv_kernel.hpp"

namespace cprune {

void launch_conv_f16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, dim3 reduce_grid) {
  launch_tile<_Float16>(tile, grid, s, a);
  if (a.split_k > 1) hipLaunchKernelGGL(splitk_reduce_kernel<_Float16>, reduce_grid, dim3(256), 0, s, a);
}

}  // namespace cprune
