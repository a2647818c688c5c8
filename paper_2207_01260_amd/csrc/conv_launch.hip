// Host side of the dense convolution: the variant table (tile x scheduling
// mode), what each variant supports and needs, and the launch.
#include "conv_ksplit_kernel.hpp"
#include "conv_pw_kernel.hpp"
#include "conv_wave_kernel.hpp"
#include "conv_stem2_kernel.hpp"
#include "conv_patch32_kernel.hpp"

namespace cprune {
namespace {

const TileVariant kTiles[] = {
#define CPRUNE_TILE_ROW(ID, WM_, WN_, MB_, NB_, KQ_) {WM_, WN_, MB_, NB_, KQ_, 1},
    CPRUNE_TILE_LIST(CPRUNE_TILE_ROW)
#undef CPRUNE_TILE_ROW
};
static_assert(sizeof(kTiles) / sizeof(kTiles[0]) == kNumTiles, "tile table");
// Scheduling modes: 0 = one output tile per work-group; n > 0 = the (tile, slab)
// work line is cut into equal runs for n * 256 resident work-groups.
const int kScheds[] = {0, 1, 2, 3, 4, 6, 8};
constexpr int kNumScheds = sizeof(kScheds) / sizeof(kScheds[0]);
constexpr int kMinUnitsPerGroup = 4;
constexpr long kMaxKsplitGroups = 8192;
constexpr int kMaxWaveMap = 32;

unsigned magic_for(unsigned d) {
  if (d <= 1) return 0;
  return (unsigned)((0x100000000ull + d - 1) / d);
}

int slab_k(int dt, int kq) { return (dt == CPRUNE_F32 ? 16 : 32) * kq; }

struct Plan {
  int tiles_m, tiles_p, slabs, units, units_per_wg, groups;
  bool fixup;
};

Plan make_plan(const cprune_conv_desc& d, const TileVariant& tv, const ConvLayout& lay) {
  Plan p;
  const int ho = conv_out_dim(d.h, d.kh, d.stride, d.pad), wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  const long P = (long)d.n * ho * wo;
  const int K = (lay.nhwc ? lay.cp_in : d.c_in) * d.kh * d.kw;
  const int kt = slab_k(d.dtype, tv.kq);
  p.tiles_m = (d.c_out + tv.tile_m() - 1) / tv.tile_m();
  p.tiles_p = (int)((P + tv.tile_p() - 1) / tv.tile_p());
  p.slabs = (K + kt - 1) / kt;
  const long units = (long)p.tiles_m * p.tiles_p * p.slabs;
  p.units = (int)units;
  if (tv.sched == 0) {
    p.units_per_wg = p.slabs;
    p.groups = p.tiles_m * p.tiles_p;
    p.fixup = false;
  } else {
    long g = (long)tv.sched * 256;
    const long cap = (units + kMinUnitsPerGroup - 1) / kMinUnitsPerGroup;
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    p.units_per_wg = (int)((units + g - 1) / g);
    p.groups = (int)((units + p.units_per_wg - 1) / p.units_per_wg);
    p.fixup = (p.units_per_wg % p.slabs) != 0;
  }
  return p;
}

}  // namespace

int num_variants() { return kNumTiles * kNumScheds + kNumPatch + kNumPatch32 + kNumKsplit + kNumPw + kNumWave + kNumPatchS2; }

namespace {
struct VariantTable {
  TileVariant table[kNumTiles * kNumScheds + kNumPatch + kNumPatch32 + kNumKsplit + kNumPw + kNumWave + kNumPatchS2];
  VariantTable() {
#define CPRUNE_PATCH_ROW(ID, MB_, TH_, TW_, NI_, KQ_, KS_)                                 \
    {                                                                         \
      TileVariant& pv = table[kNumTiles * kNumScheds + ID];                   \
      pv.wm = 1; pv.wn = 4; pv.mb = MB_; pv.nb = (TH_ * TW_ * NI_) / 64; pv.kq = KQ_; pv.ni = NI_; \
      pv.sched = -1; pv.th = TH_; pv.tw = TW_; pv.patch_id = ID; pv.ks = KS_; \
    }
    CPRUNE_PATCH_LIST(CPRUNE_PATCH_ROW)
#undef CPRUNE_PATCH_ROW
#define CPRUNE_PATCH32_ROW(ID, MB2_, NB2_, WPX_, TH_, TW_, NI_, KQ_)                       \
    {                                                                                      \
      TileVariant& pv = table[kNumTiles * kNumScheds + kNumPatch + ID];                    \
      pv.wm = 1; pv.wn = WPX_; pv.mb = 2 * MB2_; pv.nb = 2 * NB2_; pv.kq = KQ_; pv.ni = NI_; \
      pv.sched = -1; pv.th = TH_; pv.tw = TW_; pv.patch_id = ID; pv.blk32 = 1;             \
    }
    CPRUNE_PATCH32_LIST(CPRUNE_PATCH32_ROW)
#undef CPRUNE_PATCH32_ROW
#define CPRUNE_KSPLIT_ROW(ID, NB_, KW_)                                                    \
    {                                                                                      \
      TileVariant& kv = table[kNumTiles * kNumScheds + kNumPatch + kNumPatch32 + ID];      \
      kv.wm = 1; kv.wn = 1; kv.mb = 1; kv.nb = NB_; kv.kq = 1; kv.sched = -2;              \
      kv.patch_id = ID; kv.kwaves = KW_;                                                   \
    }
    CPRUNE_KSPLIT_LIST(CPRUNE_KSPLIT_ROW)
#undef CPRUNE_KSPLIT_ROW
#define CPRUNE_PW_ROW(ID, MB_, NR_)                                                        \
    {                                                                                      \
      TileVariant& kv = table[kNumTiles * kNumScheds + kNumPatch + kNumPatch32 + kNumKsplit + ID]; \
      kv.wm = 1; kv.wn = 4; kv.mb = MB_; kv.nb = 1; kv.kq = NR_; kv.sched = -3;            \
      kv.patch_id = ID; kv.nr = NR_;                                                       \
    }
    CPRUNE_PW_LIST(CPRUNE_PW_ROW)
#undef CPRUNE_PW_ROW
#define CPRUNE_WAVE_ROW(ID, NP_, NB_, KS_)                                                 \
    {                                                                                      \
      TileVariant& kv = table[kNumTiles * kNumScheds + kNumPatch + kNumPatch32 + kNumKsplit + kNumPw + ID]; \
      kv.wm = 1; kv.wn = NP_; kv.mb = 1; kv.nb = NB_; kv.kq = 1; kv.sched = -4;            \
      kv.th = 4; kv.tw = 4; kv.patch_id = ID; kv.ks = KS_;                                 \
    }
    CPRUNE_WAVE_LIST(CPRUNE_WAVE_ROW)
#undef CPRUNE_WAVE_ROW
    // (new families go behind the existing ones, so that stored variant numbers keep their meaning)
#define CPRUNE_PATCH_S2_ROW(ID, MB_, TH_, TW_, KQ_)                                        \
    {                                                                                      \
      TileVariant& pv = table[kNumTiles * kNumScheds + kNumPatch + kNumPatch32 + kNumKsplit + kNumPw + kNumWave + ID]; \
      pv.wm = 1; pv.wn = 4; pv.mb = MB_; pv.nb = (TH_ * TW_) / 64; pv.kq = KQ_; pv.ni = 1;  \
      pv.sched = -1; pv.th = TH_; pv.tw = TW_; pv.patch_id = ID; pv.stride = 2;            \
    }
    CPRUNE_PATCH_S2_LIST(CPRUNE_PATCH_S2_ROW)
#undef CPRUNE_PATCH_S2_ROW
    for (int t = 0; t < kNumTiles; ++t)
      for (int s = 0; s < kNumScheds; ++s) {
        table[t * kNumScheds + s] = kTiles[t];
        table[t * kNumScheds + s].sched = kScheds[s];
      }
  }
};
}  // namespace

const TileVariant& variant(int id) {
  static const VariantTable vt;   // built once, on first use, whichever thread gets there first
  return vt.table[id];
}

bool variant_supports(const cprune_conv_desc& d, int v, const ConvLayout& lay) {
  if (v < 0 || v >= num_variants()) return false;
  if (d.groups != 1) return false;
  const TileVariant& tv = variant(v);
  if (tv.sched == -4) {
    // 3x3 / stride 1 / pad 1 on small maps (every wavefront fetches its own weights: with many pixels the
    // tiled kernels, which share them through LDS, are the ones to use)
    if (!(lay.nhwc && lay.w_wave && d.kh == 3 && d.kw == 3 && d.stride == 1 && d.pad == 1)) return false;
    if (lay.pool == 2 || (lay.pool && ((d.h | d.w) & 1))) return false;
    if (!(d.h >= 3 && d.w >= 3 && d.h <= kMaxWaveMap && d.w <= kMaxWaveMap)) return false;
    // multiply-high divisions in the group decode: exact while groups x divisor < 2^32
    const long blocks = (long)d.n * ((d.h + 3) / 4) * ((d.w + 3) / 4);
    const long tiles_n = (blocks + tv.wn * tv.nb - 1) / (tv.wn * tv.nb);
    const long groups = tiles_n * ((d.c_out + 15) / 16);
    return groups * tiles_n < (1L << 32) && (blocks + 16) * 16 < (1L << 32);
  }
  if (tv.sched == -3) {
    // 1x1 / stride 1, no pool; exactly one (mb, nr) pair serves a shape: the smallest filter tile that
    // holds min(c_out, 128) filters and the smallest round count that holds the reduction
    if (!lay.nhwc || lay.pool || !(d.kh == 1 && d.kw == 1 && d.stride == 1 && d.pad == 0)) return false;
    const int rounds = (int)(((long)lay.cp_in * (long)dtype_size(d.dtype) + 63) / 64);
    const int nr = rounds <= 4 ? rounds : (rounds <= 6 ? 6 : 0);
    const int mb = d.c_out <= 32 ? 2 : (d.c_out <= 64 ? 4 : 8);
    return tv.nr == nr && tv.mb == mb;
  }
  if (tv.sched == -2) {
    // the reduction of a pixel is one contiguous run: 1x1 / stride 1, or a window that covers the whole map
    const bool pointwise = d.kh == 1 && d.kw == 1 && d.stride == 1 && d.pad == 0;
    const bool whole_map = d.pad == 0 && d.kh == d.h && d.kw == d.w;
    if (!lay.nhwc || !(pointwise || whole_map)) return false;
    if (lay.pool == 1 || (lay.pool == 2 && (d.c_out & 3))) return false;
    // made for few pixels: with many, the tiled kernels reuse their operands and this one does not
    const long P = (long)d.n * conv_out_dim(d.h, d.kh, d.stride, d.pad) * conv_out_dim(d.w, d.kw, d.stride, d.pad);
    const long groups = ((d.c_out + 15) / 16) * ((P + tv.tile_p() - 1) / tv.tile_p());
    return groups <= kMaxKsplitGroups;
  }
  if (tv.sched < 0) {
    if (!(lay.nhwc && d.kh == 3 && d.kw == 3 && d.stride == tv.stride && d.pad == 1)) return false;
    if (lay.pool == 2 || (lay.pool && ((d.h | d.w) & 1)) || (lay.pool && tv.stride != 1)) return false;
    const int ho = conv_out_dim(d.h, 3, d.stride, 1), wo = conv_out_dim(d.w, 3, d.stride, 1);   // = h, w at stride 1
    // multi-image tiles are for maps that fit one tile; single-image tiles for the rest
    if (tv.ni > 1 ? !(ho <= tv.th && wo <= tv.tw) : !(ho * 2 > tv.th && wo * 2 > tv.tw)) return false;
    // the kernels decode their tile with multiply-high divisions, exact while groups x divisor < 2^32
    const long tiles_s = (long)((d.n + tv.ni - 1) / tv.ni) * ((ho + tv.th - 1) / tv.th) * ((wo + tv.tw - 1) / tv.tw);
    const long groups = tiles_s * ((d.c_out + tv.tile_m() - 1) / tv.tile_m());
    return groups * tiles_s < (1L << 32);
  }
  if (lay.pool == 1) return false;                // only the patch kernels fuse a spatial pool
  if (lay.pool && lay.nhwc_out && !lay.nhwc) return false;
  if (lay.pool == 2 && !(lay.nhwc && (d.c_out & 3) == 0)) return false;
  const int ho = conv_out_dim(d.h, d.kh, d.stride, d.pad), wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  const long P = (long)d.n * ho * wo;
  const long K = (long)(lay.nhwc ? lay.cp_in : d.c_in) * d.kh * d.kw;
  const long kt = slab_k(d.dtype, tv.kq);
  const long units = ((d.c_out + tv.tile_m() - 1) / tv.tile_m()) * ((P + tv.tile_p() - 1) / tv.tile_p()) * ((K + kt - 1) / kt);
  return units < (1L << 30);
}

size_t conv_ws_bytes(const cprune_conv_desc& d, int v, const ConvLayout& lay) {
  if (d.groups != 1) return 0;
  if (v >= 0) {
    if (!variant_supports(d, v, lay)) return 0;
    const TileVariant& tv = variant(v);
    if (tv.sched < 0) return 0;
    const Plan p = make_plan(d, tv, lay);
    return p.fixup ? (size_t)2 * p.groups * tv.tile_m() * tv.tile_p() * sizeof(float) : 0;
  }
  size_t best = 0;
  for (int i = 0; i < num_variants(); ++i)
    if (variant_supports(d, i, lay)) {
      size_t b = conv_ws_bytes(d, i, lay);
      if (b > best) best = b;
    }
  return best;
}

int launch_conv_dense(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                      const void* residual, void* y, int v, void* ws, hipStream_t s, const ConvLayout& lay) {
  const TileVariant& tv = variant(v);
  const size_t es = dtype_size(d.dtype);
  if (tv.sched == -4) {
    PatchArgs pa;
    pa.x = x; pa.w = lay.w_wave; pa.bias = bias; pa.res = residual; pa.y = y;
    pa.N = d.n; pa.H = d.h; pa.W = d.w; pa.O = d.c_out; pa.Cp = lay.cp_in; pa.Cop = lay.cp_out;
    pa.pool = lay.pool;
    pa.tiles_y = (d.h + 3) / 4;
    pa.tiles_x = (d.w + 3) / 4;
    const long blocks = (long)d.n * pa.tiles_y * pa.tiles_x;
    pa.tiles_n = (int)((blocks + tv.wn * tv.nb - 1) / (tv.wn * tv.nb));   // groups along the block list
    pa.tiles_m = (d.c_out + 15) / 16;
    pa.x_bytes = (unsigned)((size_t)d.n * lay.cp_in * d.h * d.w * es);
    pa.w_bytes = (unsigned)wave_packed_bytes(d.c_out, lay.cp_in, d.dtype);
    pa.act = d.act;
    pa.vec_out = (lay.cp_out % 4) == 0 ? 1 : 0;
    pa.m_major = pa.w_bytes > pa.x_bytes ? 1 : 0;
    pa.magic_s = magic_for((unsigned)pa.tiles_n); pa.magic_m = magic_for((unsigned)pa.tiles_m);
    pa.magic_x = magic_for((unsigned)pa.tiles_x); pa.magic_y = magic_for((unsigned)pa.tiles_y);
    pa.magic_xy = magic_for((unsigned)(pa.tiles_x * pa.tiles_y));
    dim3 grid((unsigned)(pa.tiles_n * pa.tiles_m));
    int rc;
    if (d.dtype == CPRUNE_F32) rc = launch_conv_wave_f32(tv.patch_id, grid, s, pa);
    else if (d.dtype == CPRUNE_F16) rc = launch_conv_wave_f16(tv.patch_id, grid, s, pa);
    else rc = launch_conv_wave_bf16(tv.patch_id, grid, s, pa);
    if (rc != CPRUNE_OK) return rc;
    CPRUNE_LAUNCH_CHECK();
    return CPRUNE_OK;
  }
  if (tv.sched == -3) {
    ConvArgs a;
    a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.partial = nullptr;
    a.N = d.n; a.C = d.c_in; a.H = d.h; a.W = d.w; a.O = d.c_out; a.KH = 1; a.KW = 1; a.stride = 1; a.pad = 0;
    a.Ho = d.h; a.Wo = d.w;
    a.K = lay.cp_in; a.Cp = lay.cp_in; a.Cop = lay.cp_out;
    a.vec_out = (lay.cp_out % 4) == 0 ? 1 : 0;
    a.pool4 = 0; a.nhwc_out = 0;
    a.HoWo = d.h * d.w;
    a.P = d.n * a.HoWo;
    a.x_bytes = (unsigned)((size_t)a.P * lay.cp_in * es);
    a.w_bytes = (unsigned)((size_t)d.c_out * lay.cp_in * es);
    a.act = d.act;
    a.tiles_m = (d.c_out + tv.tile_m() - 1) / tv.tile_m();
    a.tiles_p = (a.P + 63) / 64;
    // persistent groups: as many as stay resident (LDS decides, at most 8 per compute unit), shared between
    // the filter tiles; each walks over its share of the pixel tiles
    const long lds = (long)tv.tile_m() * (tv.nr * 64 + 16);
    long per_cu = (160 * 1024) / lds;
    per_cu = per_cu > 8 ? 8 : (per_cu < 1 ? 1 : per_cu);
    long workers = 256 * per_cu / a.tiles_m;
    workers = workers < 1 ? 1 : (workers > a.tiles_p ? a.tiles_p : workers);
    dim3 grid((unsigned)workers, (unsigned)a.tiles_m);
    if (d.dtype == CPRUNE_F32) launch_conv_pw_f32(tv.patch_id, grid, s, a);
    else if (d.dtype == CPRUNE_F16) launch_conv_pw_f16(tv.patch_id, grid, s, a);
    else launch_conv_pw_bf16(tv.patch_id, grid, s, a);
    CPRUNE_LAUNCH_CHECK();
    return CPRUNE_OK;
  }
  if (tv.sched == -2) {
    ConvArgs a;
    a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.partial = nullptr;
    a.N = d.n; a.C = d.c_in; a.H = d.h; a.W = d.w; a.O = d.c_out; a.KH = d.kh; a.KW = d.kw;
    a.stride = d.stride; a.pad = d.pad;
    a.Ho = conv_out_dim(d.h, d.kh, d.stride, d.pad);
    a.Wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
    a.K = lay.cp_in * d.kh * d.kw;
    a.Cp = lay.cp_in; a.Cop = lay.cp_out;
    a.vec_out = (lay.cp_out % 4) == 0 ? 1 : 0;
    a.pool4 = lay.pool == 2 ? 1 : 0;
    a.nhwc_out = 0;
    a.HoWo = a.Ho * a.Wo;
    a.P = d.n * a.HoWo;
    a.x_bytes = (unsigned)((size_t)d.n * lay.cp_in * d.h * d.w * es);
    a.w_bytes = (unsigned)((size_t)d.c_out * a.K * es);
    a.act = d.act;
    a.tiles_m = (d.c_out + 15) / 16;
    a.tiles_p = (a.P + tv.tile_p() - 1) / tv.tile_p();
    a.magic_tp = magic_for((unsigned)a.tiles_p);   // at most kMaxKsplitGroups groups: exact
    if (lay.w_rows) {
      a.w = lay.w_rows;
      a.w_bytes = (unsigned)rows_packed_bytes(d.c_out, a.K, d.dtype);
      a.w_packed = 1;
    }
    dim3 grid((unsigned)(a.tiles_m * a.tiles_p));
    if (d.dtype == CPRUNE_F32) launch_conv_ksplit_f32(tv.patch_id, grid, s, a);
    else if (d.dtype == CPRUNE_F16) launch_conv_ksplit_f16(tv.patch_id, grid, s, a);
    else launch_conv_ksplit_bf16(tv.patch_id, grid, s, a);
    CPRUNE_LAUNCH_CHECK();
    return CPRUNE_OK;
  }
  if (tv.sched < 0) {
    PatchArgs pa;
    pa.x = x; pa.w = w; pa.bias = bias; pa.res = residual; pa.y = y;
    pa.N = d.n; pa.H = d.h; pa.W = d.w; pa.O = d.c_out; pa.Cp = lay.cp_in; pa.Cop = lay.cp_out;
    pa.tiles_n = (d.n + tv.ni - 1) / tv.ni;
    pa.pool = lay.pool;
    pa.Ho = conv_out_dim(d.h, 3, d.stride, 1); pa.Wo = conv_out_dim(d.w, 3, d.stride, 1);   // = h, w at stride 1
    pa.tiles_y = (pa.Ho + tv.th - 1) / tv.th;
    pa.tiles_x = (pa.Wo + tv.tw - 1) / tv.tw;
    pa.tiles_m = (d.c_out + tv.tile_m() - 1) / tv.tile_m();
    pa.x_bytes = (unsigned)((size_t)d.n * lay.cp_in * d.h * d.w * es);
    pa.w_bytes = (unsigned)((size_t)d.c_out * 9 * lay.cp_in * es);
    pa.act = d.act;
    pa.vec_out = (lay.cp_out % 4) == 0 ? 1 : 0;
    pa.m_major = pa.w_bytes > pa.x_bytes ? 1 : 0;
    pa.magic_s = magic_for((unsigned)(pa.tiles_n * pa.tiles_y * pa.tiles_x)); pa.magic_m = magic_for((unsigned)pa.tiles_m);
    pa.magic_x = magic_for((unsigned)pa.tiles_x); pa.magic_y = magic_for((unsigned)pa.tiles_y);
    pa.magic_xy = 0;
    dim3 pgrid((unsigned)(pa.tiles_n * pa.tiles_y * pa.tiles_x * pa.tiles_m));
    if (tv.stride == 2) {
      if (d.dtype == CPRUNE_F32) launch_conv_patch_s2_f32(tv.patch_id, pgrid, s, pa);
      else if (d.dtype == CPRUNE_F16) launch_conv_patch_s2_f16(tv.patch_id, pgrid, s, pa);
      else launch_conv_patch_s2_bf16(tv.patch_id, pgrid, s, pa);
    } else if (tv.blk32) {
      if (d.dtype == CPRUNE_F32) launch_conv_patch32_f32(tv.patch_id, pgrid, s, pa);
      else if (d.dtype == CPRUNE_F16) launch_conv_patch32_f16(tv.patch_id, pgrid, s, pa);
      else launch_conv_patch32_bf16(tv.patch_id, pgrid, s, pa);
    } else if (d.dtype == CPRUNE_F32) launch_conv_patch_f32(tv.patch_id, pgrid, s, pa);
    else if (d.dtype == CPRUNE_F16) launch_conv_patch_f16(tv.patch_id, pgrid, s, pa);
    else launch_conv_patch_bf16(tv.patch_id, pgrid, s, pa);
    CPRUNE_LAUNCH_CHECK();
    return CPRUNE_OK;
  }
  const Plan p = make_plan(d, tv, lay);
  ConvArgs a;
  a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.partial = (float*)ws;
  a.N = d.n; a.C = d.c_in; a.H = d.h; a.W = d.w; a.O = d.c_out; a.KH = d.kh; a.KW = d.kw;
  a.stride = d.stride; a.pad = d.pad;
  a.Ho = conv_out_dim(d.h, d.kh, d.stride, d.pad);
  a.Wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  a.K = (lay.nhwc ? lay.cp_in : d.c_in) * d.kh * d.kw;
  a.Cp = lay.cp_in;
  a.Cop = lay.cp_out;
  a.magic_cp = magic_for((unsigned)lay.cp_in);
  a.vec_out = (lay.cp_out % 4) == 0 ? 1 : 0;
  a.pool4 = lay.pool == 2 ? 1 : 0;
  a.nhwc_out = (!lay.nhwc && lay.nhwc_out) ? 1 : 0;
  a.HoWo = a.Ho * a.Wo;
  a.P = d.n * a.HoWo;
  a.HW = d.h * d.w;
  a.KHW = d.kh * d.kw;
  a.magic_khw = magic_for((unsigned)a.KHW);
  a.magic_kw = magic_for((unsigned)a.KW);
  a.x_bytes = (unsigned)((size_t)d.n * (lay.nhwc ? lay.cp_in : d.c_in) * d.h * d.w * es);
  a.w_bytes = (unsigned)((size_t)d.c_out * a.K * es);
  a.act = d.act;
  a.tiles_m = p.tiles_m;
  a.tiles_p = p.tiles_p;
  a.slabs = p.slabs;
  a.units = p.units;
  a.units_per_wg = p.units_per_wg;
  dim3 grid((unsigned)p.groups);
  const int tile = v / kNumScheds;  // implicit-GEMM variants come first in the table
  if (lay.nhwc) {
    if (d.dtype == CPRUNE_F32) launch_conv_nhwc_f32(tile, grid, s, a, p.fixup);
    else if (d.dtype == CPRUNE_F16) launch_conv_nhwc_f16(tile, grid, s, a, p.fixup);
    else launch_conv_nhwc_bf16(tile, grid, s, a, p.fixup);
  } else {
    if (d.dtype == CPRUNE_F32) launch_conv_f32(tile, grid, s, a, p.fixup);
    else if (d.dtype == CPRUNE_F16) launch_conv_f16(tile, grid, s, a, p.fixup);
    else launch_conv_bf16(tile, grid, s, a, p.fixup);
  }
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

bool conv_stem2_supported(const cprune_conv_desc& d2, const ConvLayout& lay2, int c_in, int c1) {
  if (!(c_in >= 1 && c_in <= 3 && c1 >= 1 && c1 <= 32 && d2.c_in == c1 && lay2.cp_in <= 32)) return false;
  if (!(lay2.nhwc && d2.groups == 1 && d2.kh == 3 && d2.kw == 3 && d2.stride == 1 && d2.pad == 1)) return false;
  if (d2.has_residual || lay2.pool == 2 || (lay2.pool && ((d2.h | d2.w) & 1))) return false;
  const long tiles = (long)d2.n * ((d2.h + 7) / 8) * ((d2.w + 15) / 16);
  const int mb = d2.c_out <= 16 ? 1 : (d2.c_out <= 32 ? 2 : 4);
  const long groups = tiles * ((d2.c_out + mb * 16 - 1) / (mb * 16));
  return groups * tiles < (1L << 32);   // multiply-high tile decode
}

int launch_conv_stem2(const cprune_conv_desc& d2, const ConvLayout& lay2, const void* x_nchw, int c_in,
                      const void* w1_packed, const float* b1, int c1, int act1, const void* w2, const float* b2,
                      void* y, hipStream_t s) {
  if (!conv_stem2_supported(d2, lay2, c_in, c1)) return CPRUNE_ERR_UNSUPPORTED;
  const size_t es = dtype_size(d2.dtype);
  const int mb = d2.c_out <= 16 ? 1 : (d2.c_out <= 32 ? 2 : 4);
  Stem2Args a;
  a.x = x_nchw; a.w1 = w1_packed; a.b1 = b1; a.C = c_in; a.C1 = c1; a.Cp1 = lay2.cp_in; a.act1 = act1;
  PatchArgs& pa = a.p;
  pa.x = nullptr; pa.w = w2; pa.bias = b2; pa.res = nullptr; pa.y = y;
  pa.N = d2.n; pa.H = d2.h; pa.W = d2.w; pa.O = d2.c_out; pa.Cp = lay2.cp_in; pa.Cop = lay2.cp_out;
  pa.tiles_n = d2.n;
  pa.pool = lay2.pool;
  pa.tiles_y = (d2.h + 7) / 8;
  pa.tiles_x = (d2.w + 15) / 16;
  pa.tiles_m = (d2.c_out + mb * 16 - 1) / (mb * 16);
  pa.x_bytes = 0;
  pa.w_bytes = (unsigned)((size_t)d2.c_out * 9 * lay2.cp_in * es);
  pa.act = d2.act;
  pa.vec_out = (lay2.cp_out % 4) == 0 ? 1 : 0;
  pa.m_major = 0;
  pa.magic_s = 0; pa.magic_xy = 0;
  pa.magic_m = magic_for((unsigned)pa.tiles_m);
  pa.magic_x = magic_for((unsigned)pa.tiles_x); pa.magic_y = magic_for((unsigned)pa.tiles_y);
  dim3 grid((unsigned)(pa.tiles_n * pa.tiles_y * pa.tiles_x * pa.tiles_m));
  int rc;
  if (d2.dtype == CPRUNE_F32) rc = launch_conv_stem2_f32(mb, grid, s, a);
  else if (d2.dtype == CPRUNE_F16) rc = launch_conv_stem2_f16(mb, grid, s, a);
  else rc = launch_conv_stem2_bf16(mb, grid, s, a);
  if (rc != CPRUNE_OK) return rc;
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

}  // namespace cprune
