// Instantiations of the independent-wavefront 3x3 kernel for float data.
#include "conv_wave_kernel.hpp"

namespace cprune {

int launch_conv_wave_f32(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
  return launch_wave<float>(id, grid, s, a);
}

}  // namespace cprune
