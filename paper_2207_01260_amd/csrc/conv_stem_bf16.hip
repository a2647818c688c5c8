// Instantiations of the first-layer convolution kernel for __bf16 data.
#include "conv_stem_kernel.hpp"

namespace cprune {

int launch_conv_stem_bf16(int k, int stride, int mb, dim3 grid, hipStream_t s, const StemArgs& a) {
  return launch_stem<__bf16>(k, stride, mb, grid, s, a);
}

}  // namespace cprune
