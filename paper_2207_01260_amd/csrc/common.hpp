// Shared host-side declarations of the library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bfloat16.h>
#include <stdint.h>
#include <stddef.h>

#include "cprune.h"

namespace cprune {

void set_last_hip_error(hipError_t e);

#define CPRUNE_HIP_TRY(expr)                         \
  do {                                               \
    hipError_t _e = (expr);                          \
    if (_e != hipSuccess) {                          \
      ::cprune::set_last_hip_error(_e);              \
      return CPRUNE_ERR_DEVICE;                      \
    }                                                \
  } while (0)

// Launch status check that does not synchronise.
#define CPRUNE_LAUNCH_CHECK() CPRUNE_HIP_TRY(hipGetLastError())

inline size_t dtype_size(int dt) { return dt == CPRUNE_F32 ? 4 : 2; }
inline bool dtype_ok(int dt) { return dt == CPRUNE_F32 || dt == CPRUNE_F16 || dt == CPRUNE_BF16; }
inline bool act_ok(int a) { return a == CPRUNE_ACT_NONE || a == CPRUNE_ACT_RELU || a == CPRUNE_ACT_RELU6; }

inline int conv_out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

// ---- dense conv variants -------------------------------------------------
struct TileVariant {
  int wm, wn;   // waves along output channels / pixels (wm * wn == 4)
  int mb, nb;   // 16x16 MFMA blocks per wave along channels / pixels
  int kq;       // MFMA rounds (64 bytes of k per row each) per slab
  int sched;  // scheduling mode: 0 = one tile per work-group, n = runs for n * 256 groups
  int tile_m() const { return wm * mb * 16; }
  int tile_p() const { return wn * nb * 16; }
};
int num_variants();
const TileVariant& variant(int id);

int validate_conv_desc(const cprune_conv_desc* d);
bool variant_supports(const cprune_conv_desc& d, int v);
size_t conv_ws_bytes(const cprune_conv_desc& d, int v);
int heuristic_variant(const cprune_conv_desc& d);
int cached_or_heuristic_variant(const cprune_conv_desc& d, bool* timed);
void remember_variant(const cprune_conv_desc& d, int v);

// Launchers (no argument validation: callers have validated).
int launch_conv_dense(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                      const void* residual, void* y, int v, void* ws, hipStream_t s);
int launch_conv_depthwise(const cprune_conv_desc& d, const void* x, const void* w,
                          const float* bias, const void* residual, void* y, hipStream_t s);
int launch_maxpool(const void* x, int n, int c, int h, int w, int k, int stride, int pad, int dt,
                   void* y, hipStream_t s);
int launch_gavgpool(const void* x, int n, int c, int hw, int dt, void* y, hipStream_t s);

}  // namespace cprune
