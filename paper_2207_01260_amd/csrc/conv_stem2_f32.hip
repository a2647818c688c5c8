// Instantiations of the fused first-two-layers kernel for float data.
#include "conv_stem2_kernel.hpp"

namespace cprune {

int launch_conv_stem2_f32(int mb, dim3 grid, hipStream_t s, const Stem2Args& a) {
  return launch_stem2<float>(mb, grid, s, a);
}

}  // namespace cprune
