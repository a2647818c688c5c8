// Instantiations of the fused depthwise + 1x1 projection kernel for float data.
#include "dwproj_kernel.hpp"

namespace cprune {

int launch_dwproj_f32(int k, int stride, int mb, int ks, dim3 grid, hipStream_t s, const DwProjArgs& a) {
  return launch_dwproj<float>(k, stride, mb, ks, grid, s, a);
}

}  // namespace cprune
