// Instantiations of the 16-bit 7x7 / stride 2 first-layer kernel for __bf16 data.
#include "conv_stem7_kernel.hpp"

namespace cprune {

int launch_conv_stem7_bf16(int mb, int pool, dim3 grid, hipStream_t s, const StemArgs& a) {
  return launch_stem7<__bf16>(mb, pool, grid, s, a);
}

}  // namespace cprune
