// Instantiations of the implicit-GEMM convolution kernel for __bf16 data.
#include "conv_kernel.hpp"

namespace cprune {

void launch_conv_bf16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, dim3 reduce_grid) {
  launch_tile<__bf16>(tile, grid, s, a);
  if (a.split_k > 1) hipLaunchKernelGGL(splitk_reduce_kernel<__bf16>, reduce_grid, dim3(256), 0, s, a);
}

}  // namespace cprune
