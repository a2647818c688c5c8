// Instantiations of the fused depthwise + 1x1 projection kernel for __bf16 data.
#include "dwproj_kernel.hpp"

namespace cprune {

int launch_dwproj_bf16(int k, int stride, int mb, int ks, dim3 grid, hipStream_t s, const DwProjArgs& a) {
  return launch_dwproj<__bf16>(k, stride, mb, ks, grid, s, a);
}

}  // namespace cprune
