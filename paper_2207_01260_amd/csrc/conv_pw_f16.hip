// Instantiations of the short-reduction 1x1 kernel for _Float16 data.
#include "conv_pw_kernel.hpp"

namespace cprune {

void launch_conv_pw_f16(int id, dim3 grid, hipStream_t s, const ConvArgs& a) {
  launch_pw<_Float16>(id, grid, s, a);
}

}  // namespace cprune
