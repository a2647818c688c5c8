// Host side of the dense convolution: the variant table (tile x reduction
// split), what each variant supports and needs, and the launch.
#include "conv_kernel.hpp"

namespace cprune {
namespace {

const TileVariant kTiles[] = {
#define CPRUNE_TILE_ROW(ID, WM_, WN_, MB_, NB_) {WM_, WN_, MB_, NB_, 1},
    CPRUNE_TILE_LIST(CPRUNE_TILE_ROW)
#undef CPRUNE_TILE_ROW
};
static_assert(sizeof(kTiles) / sizeof(kTiles[0]) == kNumTiles, "tile table");
const int kSplits[] = {1, 2, 4, 8, 16};
constexpr int kNumSplits = sizeof(kSplits) / sizeof(kSplits[0]);

unsigned magic_for(unsigned d) {
  if (d <= 1) return 0;
  return (unsigned)((0x100000000ull + d - 1) / d);
}

int slab_k(int dt) { return dt == CPRUNE_F32 ? 16 : 32; }

}  // namespace

int num_variants() { return kNumTiles * kNumSplits; }

const TileVariant& variant(int id) {
  static TileVariant table[kNumTiles * kNumSplits];
  static bool init = false;
  if (!init) {
    for (int t = 0; t < kNumTiles; ++t)
      for (int s = 0; s < kNumSplits; ++s) {
        table[t * kNumSplits + s] = kTiles[t];
        table[t * kNumSplits + s].split_k = kSplits[s];
      }
    init = true;
  }
  return table[id];
}

bool variant_supports(const cprune_conv_desc& d, int v) {
  if (v < 0 || v >= num_variants()) return false;
  if (d.groups != 1) return false;
  const TileVariant& tv = variant(v);
  long K = (long)d.c_in * d.kh * d.kw;
  int kt = slab_k(d.dtype);
  long slabs = (K + kt - 1) / kt;
  if (tv.split_k > 1 && slabs < 2L * tv.split_k) return false;  // at least two slabs per slice
  return true;
}

size_t conv_ws_bytes(const cprune_conv_desc& d, int v) {
  if (d.groups != 1) return 0;
  int ho = conv_out_dim(d.h, d.kh, d.stride, d.pad), wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  size_t op = (size_t)d.c_out * d.n * ho * wo * sizeof(float);
  if (v >= 0) {
    int sk = variant(v).split_k;
    return sk > 1 ? op * sk : 0;
  }
  size_t best = 0;
  for (int i = 0; i < num_variants(); ++i)
    if (variant_supports(d, i)) {
      size_t b = conv_ws_bytes(d, i);
      if (b > best) best = b;
    }
  return best;
}

int launch_conv_dense(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                      const void* residual, void* y, int v, void* ws, hipStream_t s) {
  const TileVariant& tv = variant(v);
  const size_t es = dtype_size(d.dtype);
  ConvArgs a;
  a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.partial = (float*)ws;
  a.N = d.n; a.C = d.c_in; a.H = d.h; a.W = d.w; a.O = d.c_out; a.KH = d.kh; a.KW = d.kw;
  a.stride = d.stride; a.pad = d.pad;
  a.Ho = conv_out_dim(d.h, d.kh, d.stride, d.pad);
  a.Wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  a.K = d.c_in * d.kh * d.kw;
  a.HoWo = a.Ho * a.Wo;
  a.P = d.n * a.HoWo;
  a.HW = d.h * d.w;
  a.KHW = d.kh * d.kw;
  a.magic_khw = magic_for((unsigned)a.KHW);
  a.magic_kw = magic_for((unsigned)a.KW);
  a.x_bytes = (unsigned)((size_t)d.n * d.c_in * d.h * d.w * es);
  a.w_bytes = (unsigned)((size_t)d.c_out * a.K * es);
  a.act = d.act;
  const int mt = tv.tile_m(), pt = tv.tile_p();
  a.tiles_m = (a.O + mt - 1) / mt;
  a.tiles_p = (a.P + pt - 1) / pt;
  const int kt = slab_k(d.dtype);
  const int slabs = (a.K + kt - 1) / kt;
  a.split_k = tv.split_k;
  a.k_per_split = ((slabs + tv.split_k - 1) / tv.split_k) * kt;
  dim3 grid((unsigned)(a.tiles_m * a.tiles_p), 1, (unsigned)a.split_k);
  dim3 rgrid((unsigned)(((size_t)a.O * a.P + 255) / 256));
  const int tile = v / kNumSplits;
  if (d.dtype == CPRUNE_F32) launch_conv_f32(tile, grid, s, a, rgrid);
  else if (d.dtype == CPRUNE_F16) launch_conv_f16(tile, grid, s, a, rgrid);
  else launch_conv_bf16(tile, grid, s, a, rgrid);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

}  // namespace cprune
