// Instantiations of the reduction-split dense kernel for __bf16 data.
#include "conv_ksplit_kernel.hpp"

namespace cprune {

void launch_conv_ksplit_bf16(int id, dim3 grid, hipStream_t s, const ConvArgs& a) {
  launch_ksplit<__bf16>(id, grid, s, a);
}

}  // namespace cprune
