// Instantiations of the first-layer convolution kernel for float data.
#include "conv_stem_kernel.hpp"

namespace cprune {

int launch_conv_stem_f32(int k, int stride, int mb, dim3 grid, hipStream_t s, const StemArgs& a) {
  return launch_stem<float>(k, stride, mb, grid, s, a);
}

}  // namespace cprune
