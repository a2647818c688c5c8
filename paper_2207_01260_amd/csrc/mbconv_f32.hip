// Instantiations of the fused inverted-residual block kernel for float data.
#include "mbconv_kernel.hpp"

namespace cprune {

int launch_mbconv_f32(int k, int stride, int mb, dim3 grid, size_t lds_bytes, hipStream_t s, const MbConvArgs& a) {
  return launch_mbconv<float>(k, stride, mb, grid, lds_bytes, s, a);
}

}  // namespace cprune
