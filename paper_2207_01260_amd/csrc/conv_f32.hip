// Instantiations of the implicit-GEMM convolution kernel for float data.
#include "conv_kernel.hpp"

namespace cprune {

void launch_conv_f32(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, dim3 reduce_grid) {
  launch_tile<float>(tile, grid, s, a);
  if (a.split_k > 1) hipLaunchKernelGGL(splitk_reduce_kernel<float>, reduce_grid, dim3(256), 0, s, a);
}

}  // namespace cprune
