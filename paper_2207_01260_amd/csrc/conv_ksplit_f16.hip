// Instantiations of the reduction-split dense kernel for _Float16 data.
#include "conv_ksplit_kernel.hpp"

namespace cprune {

void launch_conv_ksplit_f16(int id, dim3 grid, hipStream_t s, const ConvArgs& a) {
  launch_ksplit<_Float16>(id, grid, s, a);
}

}  // namespace cprune
