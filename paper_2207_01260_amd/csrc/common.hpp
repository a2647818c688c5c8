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
  int sched;    // scheduling mode: 0 = one tile per work-group, n = runs for n * 256 groups,
                // -1 = 3x3 spatial-patch kernel (one th x tw pixel block per work-group),
                // -2 = reduction-split kernel (16 filters x nb pixel blocks per work-group),
                // -3 = short-reduction 1x1 kernel (persistent groups, filter tile resident in LDS),
                // -4 = independent-wavefront 3x3 kernel (16 filters x wn * nb 4x4 pixel blocks x ks slices of
                //      the reduction per work-group; wn * ks wavefronts of nb blocks each)
  int th = 0, tw = 0, ni = 1, patch_id = -1;
  int blk32 = 0;  // patch kernels: 1 = 32x32 MFMA blocks (patch_id then indexes that kernel's list)
  int ks = 1;     // patch kernels on 16x16 blocks: wave groups per tile
  int kwaves = 0; // reduction-split kernel: wavefronts that share one tile's reduction (patch_id indexes its list)
  int nr = 0;     // short-reduction 1x1 kernel: 64-byte rounds of the reduction its filter tile holds
  int stride = 1; // spatial-patch kernel on 16x16 blocks: the window stride it is built for (patch_id then indexes the
                  // stride-2 list)
  int tile_m() const { return wm * mb * 16; }
  int tile_p() const { return wn * nb * 16; }
};
int num_variants();
const TileVariant& variant(int id);

// Memory layout a dense conv runs in.  nhwc = 0: NCHW activations / OIHW weights (the
// boundary's layout).  nhwc = 1: channels-last inside a network handle, channel strides
// cp_in / cp_out in elements (counts rounded up to one 16-byte vector, except a final
// dense output), weights [c_out][kh][kw][cp_in].
struct ConvLayout {
  int nhwc = 0;
  int cp_in = 0;
  int cp_out = 0;
  int nhwc_out = 0;  // with nhwc = 0: NCHW input and OIHW weights (the boundary's layout) but a channels-last
                     // output of channel stride cp_out: the first layer of a network handle
  const void* w_wave = nullptr;  // the weights once more, in the order of the independent-wavefront 3x3
                                 // kernel (launch_repack_wave); that kernel runs only where this is set
  const void* w_rows = nullptr;  // the weights once more as [16-row tile][64-byte round of the reduction][lane][16
                                 // bytes] (launch_repack_rows): the reduction-split kernel reads these when set
  int pool = 0;  // 1: channels-last 3x3 layer with a 2x2/2 max-pool fused behind the activation (patch kernels);
                 // 2: rows are (channel, position of a 2x2 map) and each group of four rows is reduced to its
                 //    maximum behind the activation; cp_out is the stride of the pooled output
};
inline int round_up_vec(int c, int dt) { const int v = dt == CPRUNE_F32 ? 4 : 8; return (c + v - 1) / v * v; }

int validate_conv_desc(const cprune_conv_desc* d);
bool variant_supports(const cprune_conv_desc& d, int v, const ConvLayout& lay = ConvLayout());
size_t conv_ws_bytes(const cprune_conv_desc& d, int v, const ConvLayout& lay = ConvLayout());
int heuristic_variant(const cprune_conv_desc& d, const ConvLayout& lay = ConvLayout());
int cached_or_heuristic_variant(const cprune_conv_desc& d, bool* timed, const ConvLayout& lay = ConvLayout());
void remember_variant(const cprune_conv_desc& d, int v, const ConvLayout& lay = ConvLayout());

// Launchers (no argument validation: callers have validated).
int launch_conv_dense(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                      const void* residual, void* y, int v, void* ws, hipStream_t s,
                      const ConvLayout& lay = ConvLayout());
int launch_conv_depthwise(const cprune_conv_desc& d, const void* x, const void* w,
                          const float* bias, const void* residual, void* y, hipStream_t s);
int launch_maxpool(const void* x, int n, int c, int h, int w, int k, int stride, int pad, int dt,
                   void* y, hipStream_t s);
int launch_gavgpool(const void* x, int n, int c, int hw, int dt, void* y, hipStream_t s);

// Channels-last layers of the network handle (cp = channel stride in elements).
int launch_depthwise_nhwc(const cprune_conv_desc& d, int cp, const void* x, const void* w_khwc,
                          const float* bias, const void* residual, void* y, hipStream_t s);
int launch_maxpool_nhwc(const void* x, int n, int cp, int h, int w, int k, int stride, int pad, int dt,
                        void* y, hipStream_t s);
int launch_gavgpool_nhwc(const void* x, int n, int cp, int hw, int dt, void* y, hipStream_t s);
int launch_nchw_to_nhwc(const void* x, int n, int c, int hw, int cp, int dt, void* y, hipStream_t s);
int launch_nhwc_to_nchw(const void* x, int n, int c, int hw, int cp, int dt, void* y, hipStream_t s);
// w [o][c][khw] -> [o][khw][cp] (zero pad); depthwise: o = 1 and c = channels gives [khw][cp]
int launch_repack_weights(const void* w, int o, int c, int khw, int cp, int dt, void* y, hipStream_t s);
// 3x3 / stride 1 / pad 1 on a 2x2 map as one matrix over the whole map: w [o][c][3][3] ->
// [rows][4 * cp_in], column (input pixel, channel), row (output pixel, channel) with channel
// stride cp_out, or (channel, output pixel) when rows_by_channel; bias [o] -> [4 * cp_out] alike
// w [o][9][cp] (channels-last 3x3 weights) -> the operand order of the independent-wavefront 3x3 kernel:
// [filter tile of 16][64-byte channel chunk][tap][lane][16 bytes], zero padded; wave_packed_bytes: its size
size_t wave_packed_bytes(int o, int cp, int dt);
int launch_repack_wave(const void* w_khwc, int o, int cp, int dt, void* y, hipStream_t s);
// w [rows][k], k contiguous -> the operand order of the reduction-split kernel, zero padded; rows_packed_bytes: size
size_t rows_packed_bytes(int rows, int k, int dt);
int launch_repack_rows(const void* w, int rows, int k, int dt, void* y, hipStream_t s);
int launch_repack_map2x2(const void* w, const float* bias, int o, int c, int cp_in, int cp_out,
                         int rows_by_channel, int dt, void* w_out, float* bias_out, hipStream_t s);

// Fused depthwise k x k (+ bias + activation) and the 1x1 convolution behind it, channels-last.
struct DwProjArgs {
  const void* x;        // [n][h][w][cpe], expanded activations
  const void* wdw;      // [k][k][cpe] depthwise weights (folded)
  const float* bdw;     // [ce] depthwise bias or null
  const void* wp;       // [o][cpe] projection weights (folded)
  const float* bp;      // [o] projection bias or null
  const void* res;      // [n][ho][wo][cop] or null
  void* y;              // [n][ho][wo][cop]
  int N, H, W, Ho, Wo, Ce, Cpe, O, Cop;
  int pad, act_dw, act_out;
  int tiles_y, tiles_x, tiles_m;
  unsigned x_bytes, wp_bytes, wdw_bytes;
  int vec_out;
};

// k in {3, 5}, stride in {1, 2}, mb in {2, 4, 8} (16-filter blocks per tile), ks in {1, 2, 4} (groups of four
// wavefronts per work-group that split the channel chunks; 4 only with k = 3 at stride 1); grid = one work-group per
// (image, 8x8 output block, filter tile).  CPRUNE_ERR_UNSUPPORTED for other combinations.
int launch_dwproj_f32(int k, int stride, int mb, int ks, dim3 grid, hipStream_t s, const DwProjArgs& a);
int launch_dwproj_f16(int k, int stride, int mb, int ks, dim3 grid, hipStream_t s, const DwProjArgs& a);
int launch_dwproj_bf16(int k, int stride, int mb, int ks, dim3 grid, hipStream_t s, const DwProjArgs& a);

// A whole inverted-residual block in one kernel: 1x1 expansion, depthwise k x k, 1x1 projection, channels-last.
struct MbConvArgs {
  const void* x;        // [n][h][w][cpi] block input
  const void* we;       // [ce][cpi] expansion weights (folded)
  const float* be;      // [ce] or null
  const void* wdw;      // [k][k][cpe] depthwise weights (folded)
  const float* bdw;     // [ce] or null
  const void* wp;       // [o][cpe] projection weights (folded)
  const float* bp;      // [o] or null
  const void* res;      // [n][ho][wo][cop] shortcut or null
  void* y;              // [n][ho][wo][cop]
  int N, H, W, Ho, Wo, Cpi, Ce, Cpe, O, Cop;
  int pad, act_e, act_dw, act_out;
  int tiles_y, tiles_x;
  unsigned x_bytes, we_bytes, wp_bytes, wdw_bytes;
  int vec_out;
  int xq;               // 16-byte quads per staged input row: cpi * sizeof(T) rounded up to 64 bytes, / 16
  unsigned magic_xq;    // division by xq
  int nchunk;           // 64-byte chunks of expanded channels
  int off_e, off_b, off_we, off_a, off_w, off_bias;   // byte offsets of the LDS regions behind the input patch
};

// LDS bytes the kernel needs (and the offsets of its regions, xq, nchunk) for a window, stride, filter
// tile (mb 16-filter blocks), input channel stride cpi, expanded channel stride cpe and element size
inline size_t mbconv_lds_layout(int k, int s, int mb, int cpi, int cpe, int es, MbConvArgs* a) {
  const int ph = 7 * s + k, npatch = ph * ph, npatchp = (npatch + 31) / 32 * 32;
  const int xrow = (cpi * es + 63) / 64 * 64 + 16, row = 64 + 16;
  const int cc = 64 / es, nchunk = (cpe + cc - 1) / cc;
  size_t off = (size_t)npatchp * xrow;
  const int off_e = (int)off; off += (size_t)2 * npatchp * row;   // double buffers of the two chunk tiles
  const int off_b = (int)off; off += (size_t)2 * 64 * row;
  const int off_we = (int)off; off += (size_t)nchunk * cc * xrow;
  const int off_a = (int)off; off += (size_t)nchunk * mb * 16 * row;
  const int off_w = (int)off; off += (size_t)nchunk * k * k * 64;
  const int off_bias = (int)off; off += (size_t)2 * nchunk * cc * sizeof(float);
  if (a) {
    a->xq = (xrow - 16) / 16;
    a->magic_xq = (unsigned)((0x100000000ull + a->xq - 1) / a->xq);
    a->nchunk = nchunk;
    a->off_e = off_e; a->off_b = off_b; a->off_we = off_we; a->off_a = off_a; a->off_w = off_w; a->off_bias = off_bias;
  }
  return off;
}

// k in {3, 5}, stride in {1, 2}, mb in {2, 4, 8} (the projection has at most 16 * mb filters); grid = persistent
// work-groups that share the (image, 8x8 output block) list round-robin; lds_bytes from mbconv_lds_layout
// (at most 160 KiB).
// CPRUNE_ERR_UNSUPPORTED for other combinations.
int launch_mbconv_f32(int k, int stride, int mb, dim3 grid, size_t lds_bytes, hipStream_t s, const MbConvArgs& a);
int launch_mbconv_f16(int k, int stride, int mb, dim3 grid, size_t lds_bytes, hipStream_t s, const MbConvArgs& a);
int launch_mbconv_bf16(int k, int stride, int mb, dim3 grid, size_t lds_bytes, hipStream_t s, const MbConvArgs& a);

// The first two layers of a network in one kernel: both 3x3 / stride 1 / pad 1, the first on the NCHW image
// (at most 3 channels) with c1 <= 32 filters, the second dense and channels-last.  d2 / lay2 describe the second
// layer (c_in = c1, cp_in = its channel stride in w2 <= 32, pool = 0 / 1); w1_packed from launch_repack_stem
// with 32 rows; y as for that layer.  CPRUNE_ERR_UNSUPPORTED outside these limits.
bool conv_stem2_supported(const cprune_conv_desc& d2, const ConvLayout& lay2, int c_in, int c1);
int launch_conv_stem2(const cprune_conv_desc& d2, const ConvLayout& lay2, const void* x_nchw, int c_in,
                      const void* w1_packed, const float* b1, int c1, int act1, const void* w2, const float* b2,
                      void* y, hipStream_t s);

// First-layer convolution: NCHW input with at most 3 channels, OIHW weights, channels-last output.
struct StemArgs {
  const void* x;        // [n][c][h][w]
  const void* w;        // [tiles_m * 16 * mb][kp] packed by launch_repack_stem: k = (c, u, v) padded with
                        // zeros to kp, rows beyond o zero
  const float* bias;    // [o] or null
  void* y;              // [n][ho][wo][cop]
  int N, C, H, W, Ho, Wo, O, Cop;
  int pad, act;
  int tiles_y, tiles_x, tiles_m;
  unsigned magic_x, magic_y;   // ceil(2^32 / tiles_x), ceil(2^32 / tiles_y), 0 for a divisor of 1 (exact while
                               // pixel blocks x divisor < 2^32: always, for tensors below 2^31 bytes)
  int vec_out;
  int Hp = 0, Wp = 0;   // 7x7 / stride 2 kernel with the 3x3 / stride 2 / pad 1 max-pool inside: the pooled map; y is
                        // then [n][hp][wp][cop] and tiles_y, tiles_x count 7 x 7 blocks of it
};
// (k, stride) in {(3, 1), (3, 2), (7, 2)}, mb in {2, 4} (16-filter blocks per tile); grid.x = workers
// that share the (image, 8x16 output block) list round-robin, grid.y = filter tiles.
// CPRUNE_ERR_UNSUPPORTED for other windows.  stem_packed_k: padded row length in elements.
int stem_packed_k(int k, int dt);
int launch_repack_stem(const void* w, int o, int ktot, int rows, int kp, int dt, void* y, hipStream_t s);
int launch_conv_stem_f32(int k, int stride, int mb, dim3 grid, hipStream_t s, const StemArgs& a);
int launch_conv_stem_f16(int k, int stride, int mb, dim3 grid, hipStream_t s, const StemArgs& a);
int launch_conv_stem_bf16(int k, int stride, int mb, dim3 grid, hipStream_t s, const StemArgs& a);
// 16-bit 7x7 / stride 2 / pad 3 first layer with the reduction ordered (window row, 8 window columns, 4 channels):
// weights [rows][224] from launch_repack_stem7 (k = u * 32 + (v + 1) * 4 + c; zero for column slot 0, channel
// slot 3, channels beyond c and rows beyond o).  mb in {2, 4}; pool = 1 runs the 3x3 / stride 2 / pad 1 max-pool
// too (StemArgs::Hp, Wp); grid.x = workers sharing the (image, block) list, grid.y = filter tiles.
constexpr int kStem7K = 224;
int launch_repack_stem7(const void* w, int o, int c, int rows, int dt, void* y, hipStream_t s);
int launch_conv_stem7_f16(int mb, int pool, dim3 grid, hipStream_t s, const StemArgs& a);
int launch_conv_stem7_bf16(int mb, int pool, dim3 grid, hipStream_t s, const StemArgs& a);

}  // namespace cprune
