// Instantiations of the reduction-split dense kernel for float data.
#include "conv_ksplit_kernel.hpp"

namespace cprune {

void launch_conv_ksplit_f32(int id, dim3 grid, hipStream_t s, const ConvArgs& a) {
  launch_ksplit<float>(id, grid, s, a);
}

}  // namespace cprune
