// Instantiations of the fused first-two-layers kernel for _Float16 data.
#include "conv_stem2_kernel.hpp"

namespace cprune {

int launch_conv_stem2_f16(int mb, dim3 grid, hipStream_t s, const Stem2Args& a) {
  return launch_stem2<_Float16>(mb, grid, s, a);
}

}  // namespace cprune
