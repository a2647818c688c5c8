// Instantiations of the independent-wavefront 3x3 kernel for __bf16 data.
#include "conv_wave_kernel.hpp"

namespace cprune {

int launch_conv_wave_bf16(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
  return launch_wave<__bf16>(id, grid, s, a);
}

}  // namespace cprune
