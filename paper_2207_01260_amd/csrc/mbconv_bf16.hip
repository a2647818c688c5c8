// Instantiations of the fused inverted-residual block kernel for __bf16 data.
#include "mbconv_kernel.hpp"

namespace cprune {

int launch_mbconv_bf16(int k, int stride, int mb, dim3 grid, size_t lds_bytes, hipStream_t s, const MbConvArgs& a) {
  return launch_mbconv<__bf16>(k, stride, mb, grid, lds_bytes, s, a);
}

}  // namespace cprune
