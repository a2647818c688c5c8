// C-ABI entry points: argument validation, the per-shape variant cache and
// on-device selection, the single-layer calls and the network handle.
#include "common.hpp"

#include <map>
#include <mutex>
#include <vector>
#include <algorithm>
#include <array>
#include <cmath>
#include <cstdio>
#include <cstring>

namespace cprune {

static thread_local hipError_t g_last_hip_error = hipSuccess;
void set_last_hip_error(hipError_t e) { g_last_hip_error = e; }

// ---- descriptor validation ---------------------------------------------------
int validate_conv_desc(const cprune_conv_desc* d) {
  if (!d) return CPRUNE_ERR_INVALID_ARG;
  if (d->n < 1 || d->c_in < 1 || d->h < 1 || d->w < 1 || d->c_out < 1) return CPRUNE_ERR_INVALID_ARG;
  if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0) return CPRUNE_ERR_INVALID_ARG;
  if (!dtype_ok(d->dtype) || !act_ok(d->act)) return CPRUNE_ERR_INVALID_ARG;
  if (d->has_residual != 0 && d->has_residual != 1) return CPRUNE_ERR_INVALID_ARG;
  if (d->groups < 1) return CPRUNE_ERR_INVALID_ARG;
  if (d->h + 2 * d->pad < d->kh || d->w + 2 * d->pad < d->kw) return CPRUNE_ERR_INVALID_ARG;
  if (d->groups != 1 && !(d->groups == d->c_in && d->c_out == d->c_in)) return CPRUNE_ERR_UNSUPPORTED;
  if (d->kh > 7 || d->kw > 7) return CPRUNE_ERR_UNSUPPORTED;
  if (d->pad >= d->kh || d->pad >= d->kw) return CPRUNE_ERR_UNSUPPORTED;  // every window holds a real element
  const long ho = conv_out_dim(d->h, d->kh, d->stride, d->pad), wo = conv_out_dim(d->w, d->kw, d->stride, d->pad);
  const long lim = 1L << 31;
  if (d->groups == 1) {  // the dense kernel addresses x and w with 31-bit byte offsets
    const long es = (long)dtype_size(d->dtype);
    if ((long)d->n * d->c_in * d->h * d->w * es >= lim) return CPRUNE_ERR_UNSUPPORTED;
    if ((long)d->c_out * d->c_in * d->kh * d->kw * es >= lim) return CPRUNE_ERR_UNSUPPORTED;
  }
  if ((long)d->n * d->c_in * d->h * d->w >= lim || (long)d->n * d->c_out * ho * wo >= lim) return CPRUNE_ERR_UNSUPPORTED;
  if ((long)d->c_out * (d->c_in / d->groups) * d->kh * d->kw >= lim) return CPRUNE_ERR_UNSUPPORTED;
  if ((long)d->c_in * d->kh * d->kw * d->kh * d->kw >= lim) return CPRUNE_ERR_UNSUPPORTED;  // exact magic division
  return CPRUNE_OK;
}

// ---- variant cache -------------------------------------------------------------
typedef std::array<int, 18> DescKey;
static DescKey key_of(const cprune_conv_desc& d, const ConvLayout& lay) {
  return DescKey{d.n, d.c_in, d.h, d.w, d.c_out, d.kh, d.kw, d.stride, d.pad, d.groups, d.dtype, d.act,
                 d.has_residual, lay.nhwc, lay.cp_in, lay.cp_out, lay.pool, lay.nhwc_out};
}
static std::mutex g_cache_mutex;
static std::map<DescKey, int> g_cache;

void remember_variant(const cprune_conv_desc& d, int v, const ConvLayout& lay) {
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  g_cache[key_of(d, lay)] = v;
}

// Untimed fallback: the tile whose wavefronts reuse their LDS operands most (blocks
// per operand fetched), discounted by the pixel columns a ragged last tile wastes;
// work cut into equal runs for 512 resident work-groups, which needs no knowledge
// of how the tile count divides the chip.  Used only for shapes never timed.
int heuristic_variant(const cprune_conv_desc& d, const ConvLayout& lay) {
  const long ho = conv_out_dim(d.h, d.kh, d.stride, d.pad), wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  const long P = (long)d.n * ho * wo, O = d.c_out;
  double best = -1.0;
  int best_v = 0;
  for (int v = 0; v < num_variants(); ++v) {
    const TileVariant& tv = variant(v);
    if (tv.sched != 2 || !variant_supports(d, v, lay)) continue;
    const long mt = tv.tile_m(), pt = tv.tile_p();
    const long tm = (O + mt - 1) / mt, tp = (P + pt - 1) / pt;
    double rows16 = std::ceil((double)O / tm / 16.0 / tv.wm);
    if (rows16 > tv.mb) rows16 = tv.mb;
    const double reuse = rows16 * tv.nb / (rows16 + tv.nb);
    const double fill = (double)P / (double)(tp * pt);
    const double score = reuse * fill;
    if (score > best) { best = score; best_v = v; }
  }
  if (best < 0.0)  // nothing among the cut-run variants (a fused pool needs a patch kernel): first that runs
    for (int v = 0; v < num_variants(); ++v)
      if (variant_supports(d, v, lay)) return v;
  return best_v;
}

int cached_or_heuristic_variant(const cprune_conv_desc& d, bool* timed, const ConvLayout& lay) {
  {
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    auto it = g_cache.find(key_of(d, lay));
    if (it != g_cache.end()) {
      if (timed) *timed = true;
      return it->second;
    }
  }
  if (timed) *timed = false;
  return heuristic_variant(d, lay);
}

static int conv_dispatch(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                         const void* residual, void* y, int v, void* ws, size_t ws_bytes, hipStream_t s,
                         const ConvLayout& lay = ConvLayout()) {
  if (d.groups != 1)
    return lay.nhwc ? launch_depthwise_nhwc(d, lay.cp_in, x, w, bias, residual, y, s)
                    : launch_conv_depthwise(d, x, w, bias, residual, y, s);
  if (v < 0) v = cached_or_heuristic_variant(d, nullptr, lay);
  if (!variant_supports(d, v, lay)) return CPRUNE_ERR_UNSUPPORTED;
  const size_t need = conv_ws_bytes(d, v, lay);
  if (need > 0 && (!ws || ws_bytes < need)) return CPRUNE_ERR_WORKSPACE;
  return launch_conv_dense(d, x, w, bias, residual, y, v, ws, s, lay);
}

// Times every supported variant on the given buffers; returns the fastest.  Two stages: every
// variant briefly, then the few best again with more repetitions, so that a short disturbance
// (another process's burst, a clock change) during one measurement does not decide the choice.
static int select_tile_impl(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                            const void* residual, void* y, void* ws, size_t ws_bytes, int warmup,
                            int iters, int* variant_out, float* best_ms_out, float* all_ms_out,
                            hipStream_t s, const ConvLayout& lay = ConvLayout()) {
  hipEvent_t e0, e1;
  CPRUNE_HIP_TRY(hipEventCreate(&e0));
  hipError_t ee = hipEventCreate(&e1);
  if (ee != hipSuccess) { hipEventDestroy(e0); set_last_hip_error(ee); return CPRUNE_ERR_DEVICE; }
  int rc = CPRUNE_OK;
  // fastest of `passes` timed passes of `n` launches each, per launch
  auto time_variant = [&](int v, int n, int passes, float* ms_out) -> int {
    float ms = 0.0f;
    for (int pass = 0; pass < passes; ++pass) {
      int r = CPRUNE_OK;
      hipError_t e = hipEventRecord(e0, s);
      for (int i = 0; i < n && r == CPRUNE_OK; ++i) r = conv_dispatch(d, x, w, bias, residual, y, v, ws, ws_bytes, s, lay);
      if (r != CPRUNE_OK) return r;
      if (e == hipSuccess) e = hipEventRecord(e1, s);
      if (e == hipSuccess) e = hipEventSynchronize(e1);
      float t = 0.0f;
      if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
      if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
      t /= (float)n;
      if (pass == 0 || t < ms) ms = t;
    }
    *ms_out = ms;
    return CPRUNE_OK;
  };
  std::vector<std::pair<float, int>> timed;
  int supported = d.groups == 1 ? 0 : 1;   // variants that can run the shape (timed or not)
  const int nv = d.groups == 1 ? num_variants() : 1;
  for (int v = 0; v < nv && rc == CPRUNE_OK; ++v) {
    if (all_ms_out) all_ms_out[v] = -1.0f;
    if (d.groups == 1) {
      if (!variant_supports(d, v, lay)) continue;
      ++supported;
      if (conv_ws_bytes(d, v, lay) > ws_bytes) continue;  // not timed: the caller's scratch cannot run it
    }
    for (int i = 0; i < warmup && rc == CPRUNE_OK; ++i) rc = conv_dispatch(d, x, w, bias, residual, y, v, ws, ws_bytes, s, lay);
    if (rc != CPRUNE_OK) break;
    float ms = 0.0f;
    rc = time_variant(v, iters, 2, &ms);
    if (rc != CPRUNE_OK) break;
    if (all_ms_out) all_ms_out[v] = ms;
    timed.emplace_back(ms, v);
  }
  if (rc == CPRUNE_OK && timed.size() > 1) {
    std::sort(timed.begin(), timed.end());
    const size_t finalists = timed.size() < 4 ? timed.size() : 4;
    for (size_t k = 0; k < finalists && rc == CPRUNE_OK; ++k) {
      float ms = 0.0f;
      rc = time_variant(timed[k].second, 3 * iters, 3, &ms);
      if (rc != CPRUNE_OK) break;
      timed[k].first = ms;
      if (all_ms_out) all_ms_out[timed[k].second] = timed[k].first;
    }
    std::sort(timed.begin(), timed.begin() + finalists);
  }
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  if (rc != CPRUNE_OK) return rc;
  if (timed.empty()) return supported ? CPRUNE_ERR_WORKSPACE : CPRUNE_ERR_UNSUPPORTED;
  const int best_v = timed[0].second;
  if (d.groups == 1) remember_variant(d, best_v, lay);
  if (variant_out) *variant_out = best_v;
  if (best_ms_out) *best_ms_out = timed[0].first;
  return CPRUNE_OK;
}

}  // namespace cprune

using namespace cprune;

extern "C" const char* cprune_status_string(int status) {
  switch (status) {
    case CPRUNE_OK: return "ok";
    case CPRUNE_ERR_INVALID_ARG: return "invalid argument";
    case CPRUNE_ERR_UNSUPPORTED: return "unsupported configuration";
    case CPRUNE_ERR_WORKSPACE: return "workspace too small";
    case CPRUNE_ERR_DEVICE: return "HIP call failed";
    case CPRUNE_ERR_NOT_TUNED: return "shape not tuned";
    default: return "unknown status";
  }
}

extern "C" int cprune_last_hip_error(void) { return (int)g_last_hip_error; }

extern "C" int cprune_num_tile_variants(void) { return num_variants(); }

extern "C" int cprune_tile_variant_info(int v, int* tile_m, int* tile_p, int* sched) {
  if (v < 0 || v >= num_variants()) return CPRUNE_ERR_INVALID_ARG;
  const TileVariant& tv = variant(v);
  if (tile_m) *tile_m = tv.tile_m();
  if (tile_p) *tile_p = tv.tile_p();
  if (sched) *sched = tv.sched;
  return CPRUNE_OK;
}

extern "C" int cprune_tile_variant_name(int v, int channels_last, cprune_dtype dtype, char* buf, size_t buf_bytes) {
  if (v < 0 || v >= num_variants() || !buf || buf_bytes < 1 || !dtype_ok(dtype)) return CPRUNE_ERR_INVALID_ARG;
  const TileVariant& tv = variant(v);
  const char* t = dtype == CPRUNE_F32 ? "float" : dtype == CPRUNE_F16 ? "_Float16" : "__bf16";
  int n;
  if (tv.sched >= 0)
    n = snprintf(buf, buf_bytes, "%s<%s, %d, %d, %d, %d, %d>", channels_last ? "conv_nhwc_kernel" : "conv_igemm_kernel", t,
                 tv.wm, tv.wn, tv.mb, tv.nb, tv.kq);
  else if (tv.sched == -4)
    n = snprintf(buf, buf_bytes, "conv_wave_kernel<%s, %d, %d, %d>", t, tv.wn, tv.nb, tv.ks);
  else if (tv.sched == -3)
    n = snprintf(buf, buf_bytes, "conv_pw_kernel<%s, %d, %d>", t, tv.mb, tv.nr);
  else if (tv.sched == -2)
    n = snprintf(buf, buf_bytes, "conv_ksplit_kernel<%s, %d, %d>", t, tv.nb, tv.kwaves);
  else if (tv.blk32)
    n = snprintf(buf, buf_bytes, "conv_patch32_kernel<%s, %d, %d, %d, %d, %d, %d, %d>", t, tv.mb / 2, tv.nb / 2, tv.wn, tv.th,
                 tv.tw, tv.ni, tv.kq);
  else if (tv.stride == 2)
    n = snprintf(buf, buf_bytes, "conv_patch_s2_kernel<%s, %d, %d, %d, %d>", t, tv.mb, tv.th, tv.tw, tv.kq);
  else
    n = snprintf(buf, buf_bytes, "conv_patch_kernel<%s, %d, %d, %d, %d, %d, %d>", t, tv.mb, tv.th, tv.tw, tv.ni, tv.kq, tv.ks);
  return (n < 0 || (size_t)n >= buf_bytes) ? CPRUNE_ERR_INVALID_ARG : CPRUNE_OK;
}

extern "C" size_t cprune_conv_workspace_bytes(const cprune_conv_desc* desc, int v) {
  if (validate_conv_desc(desc) != CPRUNE_OK) return 0;
  if (v >= num_variants()) return 0;
  return conv_ws_bytes(*desc, v);
}

extern "C" int cprune_conv2d_bn_relu(const cprune_conv_desc* desc, const void* x, const void* w,
                                     const float* bias, const void* residual, void* y, int tile_variant,
                                     void* ws, size_t ws_bytes, void* stream) {
  int rc = validate_conv_desc(desc);
  if (rc != CPRUNE_OK) return rc;
  if (!x || !w || !y) return CPRUNE_ERR_INVALID_ARG;
  if ((desc->has_residual != 0) != (residual != nullptr)) return CPRUNE_ERR_INVALID_ARG;
  if (tile_variant < -1 || tile_variant >= num_variants()) return CPRUNE_ERR_INVALID_ARG;
  return conv_dispatch(*desc, x, w, bias, residual, y, tile_variant, ws, ws_bytes, (hipStream_t)stream);
}

extern "C" int cprune_select_tile(const cprune_conv_desc* desc, const void* x, const void* w,
                                  const float* bias, const void* residual, void* y, void* ws,
                                  size_t ws_bytes, int warmup, int iters, int* variant_out,
                                  float* best_ms_out, float* all_ms_out, void* stream) {
  int rc = validate_conv_desc(desc);
  if (rc != CPRUNE_OK) return rc;
  if (!x || !w || !y || !variant_out) return CPRUNE_ERR_INVALID_ARG;
  if ((desc->has_residual != 0) != (residual != nullptr)) return CPRUNE_ERR_INVALID_ARG;
  if (warmup < 0 || iters < 1) return CPRUNE_ERR_INVALID_ARG;
  return select_tile_impl(*desc, x, w, bias, residual, y, ws, ws ? ws_bytes : 0, warmup, iters, variant_out,
                          best_ms_out, all_ms_out, (hipStream_t)stream);
}

extern "C" void cprune_clear_tile_cache(void) {
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  g_cache.clear();
}

extern "C" int cprune_cached_tile(const cprune_conv_desc* desc, int* variant_out, int* was_timed_out) {
  int rc = validate_conv_desc(desc);
  if (rc != CPRUNE_OK) return rc;
  if (!variant_out) return CPRUNE_ERR_INVALID_ARG;
  if (desc->groups != 1) return CPRUNE_ERR_UNSUPPORTED;
  bool timed = false;
  *variant_out = cached_or_heuristic_variant(*desc, &timed);
  if (was_timed_out) *was_timed_out = timed ? 1 : 0;
  return CPRUNE_OK;
}

extern "C" int cprune_maxpool2d(const void* x, int n, int c, int h, int w, int k, int stride, int pad,
                                cprune_dtype dtype, void* y, void* stream) {
  if (!x || !y || n < 1 || c < 1 || h < 1 || w < 1 || k < 1 || stride < 1 || pad < 0) return CPRUNE_ERR_INVALID_ARG;
  if (!dtype_ok(dtype) || h + 2 * pad < k || w + 2 * pad < k) return CPRUNE_ERR_INVALID_ARG;
  if (pad >= k) return CPRUNE_ERR_UNSUPPORTED;
  if ((long)n * c * h * w >= (1L << 31)) return CPRUNE_ERR_UNSUPPORTED;
  return launch_maxpool(x, n, c, h, w, k, stride, pad, dtype, y, (hipStream_t)stream);
}

extern "C" int cprune_global_avgpool(const void* x, int n, int c, int h, int w, cprune_dtype dtype,
                                     void* y, void* stream) {
  if (!x || !y || n < 1 || c < 1 || h < 1 || w < 1 || !dtype_ok(dtype)) return CPRUNE_ERR_INVALID_ARG;
  if ((long)n * c * h * w >= (1L << 31)) return CPRUNE_ERR_UNSUPPORTED;
  return launch_gavgpool(x, n, c, h * w, dtype, y, (hipStream_t)stream);
}

static cprune_conv_desc fc_desc(int n, int f, int c_out, int act, int dtype) {
  cprune_conv_desc d;
  d.n = n; d.c_in = f; d.h = 1; d.w = 1; d.c_out = c_out; d.kh = 1; d.kw = 1; d.stride = 1; d.pad = 0;
  d.groups = 1; d.dtype = dtype; d.act = act; d.has_residual = 0;
  return d;
}

extern "C" size_t cprune_fc_workspace_bytes(int n, int f, int c_out, cprune_dtype dtype) {
  if (n < 1 || f < 1 || c_out < 1 || !dtype_ok(dtype)) return 0;
  cprune_conv_desc d = fc_desc(n, f, c_out, CPRUNE_ACT_NONE, dtype);
  return conv_ws_bytes(d, -1);
}

extern "C" int cprune_fc(const void* x, const void* w, const float* bias, int n, int f, int c_out,
                         cprune_act act, cprune_dtype dtype, void* y, void* ws, size_t ws_bytes,
                         void* stream) {
  if (n < 1 || f < 1 || c_out < 1 || !x || !w || !y) return CPRUNE_ERR_INVALID_ARG;
  if (!dtype_ok(dtype) || !act_ok(act)) return CPRUNE_ERR_INVALID_ARG;
  cprune_conv_desc d = fc_desc(n, f, c_out, act, dtype);
  int rc = validate_conv_desc(&d);
  if (rc != CPRUNE_OK) return rc;
  // the remembered or heuristic variant, or its one-tile-per-group twin when the
  // caller's scratch is too small for cut tiles
  int v = cached_or_heuristic_variant(d, nullptr);
  if (conv_ws_bytes(d, v) > (ws ? ws_bytes : 0)) {
    int twin = -1;
    for (int i = 0; i < num_variants(); ++i)
      if (variant_supports(d, i) && variant(i).sched == 0 && variant(i).tile_m() == variant(v).tile_m() &&
          variant(i).tile_p() == variant(v).tile_p()) { twin = i; break; }
    if (twin < 0) return CPRUNE_ERR_WORKSPACE;
    v = twin;
  }
  return launch_conv_dense(d, x, w, bias, nullptr, y, v, ws, (hipStream_t)stream);
}

// ---- network handle ------------------------------------------------------------
// Inside a handle everything is channels-last: activations [n][h][w][cp], dense weights
// [c_out][kh][kw][cp], depthwise weights [kh][kw][cp], with cp the channel count rounded up
// to one 16-byte vector (pad channels are zero and stay zero through every layer).  The
// boundary stays NCHW: a dense first layer with few input channels reads the caller's tensor
// as it is (any other reader gets a converted copy); activations are converted on the way out.
struct NetLayer {
  cprune_layer_desc d;
  int h_in, w_in, h_out, w_out;
  int cp_in = 0, cp_out = 0;  // channel strides of the input / output buffers
  void* w = nullptr;
  float* b = nullptr;
  void* act = nullptr;        // [max_batch][h_out][w_out][cp_out]
  size_t per_image = 0;       // elements per image of the output buffer
  int variant = -1;           // dense conv / fc: variant for max_batch
  bool fused_pool = false;    // conv: the 2x2 max-pool that follows runs in its epilogue; act is the pooled map
  bool alias = false;         // max-pool folded into its producer: no kernel, act is the producer's buffer
  bool map2x2 = false;        // 3x3 / stride 1 / pad 1 conv on a 2x2 map, run as one matrix over the whole map
  int fuse_dw = -1;           // 1x1 conv: index of the depthwise layer computed inside its kernel, or -1
  int dw_ks = 1;              // ... and how many groups of four wavefronts share one pixel block there
  bool fused_away = false;    // depthwise conv that runs inside its consumer's kernel (no launch, no activation)
  int dw_reader = -1;         // depthwise conv that may run inside the 1x1 conv dw_reader's kernel
  int fuse_block = -1;        // 1x1 conv with fuse_dw set: index of the 1x1 expansion in front of that depthwise
                              // layer when the whole block (expansion, depthwise, this projection) is one kernel
  int block_expand = -1;      // depthwise conv: the expansion layer that may join it and dw_reader in one kernel
  int fuse_stem = -1;         // 3x3 conv: index of the first layer (on the image) computed inside its kernel, or -1
  int stem_reader = -1;       // first layer that may run inside the 3x3 conv stem_reader's kernel
  void* w_stem = nullptr;     // weights packed for the first-layer kernel
  void* w_rows = nullptr;     // layer the reduction-split kernel can run: weights once more, in its operand order
  void* w_wave = nullptr;     // 3x3 / stride 1 / pad 1 layer on a small map: weights once more, packed for the
                              // independent-wavefront kernel
  bool stem = false;          // nchw_in layer that runs the first-layer kernel (whole reduction in LDS)
  void* w_stem7 = nullptr;    // 16-bit 7x7 / stride 2 / pad 3 first layer: weights packed for the kernel made for it
  int stem7 = 0;              // 1: that kernel runs the layer; 2: and the 3x3 / stride 2 max-pool pool3 with it
  int pool3 = -1;             // the max-pool that can run inside that kernel (the layer's only reader), or -1
  bool in_producer = false;   // max-pool computed inside its producer's kernel: no launch, its buffer is written there
  int stem_ok = 0;            // that kernel exists for the layer's window and stride
  bool nchw_in = false;       // dense conv on the network input: reads the caller's NCHW tensor and its own
                              // OIHW weights, writes channels-last (no layout conversion pass)
};

struct GraphKey {
  int n; const void* x; void* logits;
  bool operator<(const GraphKey& o) const {
    if (n != o.n) return n < o.n;
    if (x != o.x) return x < o.x;
    return logits < o.logits;
  }
};

struct cprune_net {
  std::vector<NetLayer> layers;
  int in_c, in_h, in_w, in_cp, max_batch, dtype;
  std::vector<void*> allocs;
  void* x_cl = nullptr;       // the network input, channels-last
  bool convert_input = true;  // false when every reader of the input takes the caller's NCHW tensor itself
  void* ws = nullptr;
  size_t ws_bytes = 0;
  struct GraphEntry { hipGraphExec_t exec; uint64_t last_use; };
  std::map<GraphKey, GraphEntry> graphs;   // at most kMaxGraphs: the least recently used one makes room
  uint64_t graph_clock = 0;
  hipStream_t capture_stream = nullptr;  // graphs are recorded here (the caller's may be the null stream)
  int last_n = 0;
};

// A fully connected layer is a convolution whose kernel covers its whole input map.
static cprune_conv_desc layer_conv_desc(const cprune_net& net, const NetLayer& L, int n) {
  cprune_conv_desc d;
  d.n = n; d.c_in = L.d.c_in; d.c_out = L.d.c_out; d.dtype = net.dtype; d.act = L.d.act;
  d.has_residual = L.d.residual >= 0 ? 1 : 0;
  d.h = L.h_in; d.w = L.w_in;
  if (L.map2x2) {
    // channels-last, a 2x2 map of cp channels is one vector of 4 * cp values per image
    d.c_in = 4 * L.cp_in; d.c_out = 4 * round_up_vec(L.d.c_out, net.dtype);
    d.h = d.w = 1; d.kh = d.kw = 1; d.stride = 1; d.pad = 0; d.groups = 1;
    return d;
  }
  if (L.d.kind == CPRUNE_LAYER_FC) {
    d.kh = L.h_in; d.kw = L.w_in; d.stride = 1; d.pad = 0; d.groups = 1;
  } else {
    d.kh = d.kw = L.d.k; d.stride = L.d.stride; d.pad = L.d.pad; d.groups = L.d.groups;
  }
  return d;
}

static ConvLayout layer_layout(const NetLayer& L) {
  ConvLayout lay;
  lay.nhwc = 1; lay.cp_in = L.cp_in; lay.cp_out = L.cp_out; lay.pool = L.fused_pool ? 1 : 0;
  lay.w_wave = L.w_wave;
  lay.w_rows = L.w_rows;
  if (L.nchw_in) { lay.nhwc = 0; lay.nhwc_out = 1; lay.cp_in = 0; return lay; }
  if (L.map2x2) {
    lay.cp_in = 4 * L.cp_in;
    if (L.fused_pool) lay.pool = 2;   // rows ordered (channel, pixel); cp_out stays the pooled map's stride
    else lay.cp_out = 4 * L.cp_out;
  }
  return lay;
}

constexpr size_t kMaxGraphs = 8;

static void drop_graphs(cprune_net* net) {
  for (auto& g : net->graphs) hipGraphExecDestroy(g.second.exec);
  net->graphs.clear();
}

static void net_free(cprune_net* net) {
  drop_graphs(net);
  if (net->capture_stream) hipStreamDestroy(net->capture_stream);
  for (void* p : net->allocs) hipFree(p);
  delete net;
}

// The first-layer kernel on the caller's NCHW input.
static int net_run_stem(cprune_net* net, int i, int n, const void* x, void* dst, hipStream_t s) {
  const NetLayer& L = net->layers[i];
  StemArgs a;
  a.x = x; a.w = L.w_stem; a.bias = L.b; a.y = dst;
  a.N = n; a.C = L.d.c_in; a.H = L.h_in; a.W = L.w_in; a.Ho = L.h_out; a.Wo = L.w_out;
  a.O = L.d.c_out; a.Cop = L.cp_out; a.pad = L.d.pad; a.act = L.d.act;
  const int mb = L.d.c_out <= 32 ? 2 : 4;
  a.tiles_y = (a.Ho + 7) / 8; a.tiles_x = (a.Wo + 15) / 16; a.tiles_m = (a.O + mb * 16 - 1) / (mb * 16);
  a.vec_out = (a.Cop % 4) == 0 ? 1 : 0;
  a.magic_x = a.tiles_x > 1 ? (unsigned)((0x100000000ull + a.tiles_x - 1) / a.tiles_x) : 0u;
  a.magic_y = a.tiles_y > 1 ? (unsigned)((0x100000000ull + a.tiles_y - 1) / a.tiles_y) : 0u;
  const long ptiles = (long)n * a.tiles_y * a.tiles_x;
  // as many workers as stay resident: LDS per work-group = weight tile + patch + offset table
  const int es = (int)dtype_size(net->dtype), kp = stem_packed_k(L.d.k, net->dtype);
  const int ph = 7 * L.d.stride + L.d.k, pwp = (15 * L.d.stride + L.d.k + 3) / 4 * 4;
  const long lds = (long)mb * 16 * (kp * es + 16) + 3L * ph * pwp * es + kp * 4;
  long per_cu = (160 * 1024) / lds;
  per_cu = per_cu > 8 ? 8 : (per_cu < 1 ? 1 : per_cu);
  // a small weight tile costs little to stage: then one pixel block per work-group keeps more of them in flight
  const bool light = (long)mb * 16 * (kp * es + 16) < 8192;
  const long workers = (light || ptiles < 256 * per_cu) ? ptiles : 256 * per_cu;
  dim3 grid((unsigned)workers, (unsigned)a.tiles_m);
  int rc;
  if (net->dtype == CPRUNE_F32) rc = launch_conv_stem_f32(L.d.k, L.d.stride, mb, grid, s, a);
  else if (net->dtype == CPRUNE_F16) rc = launch_conv_stem_f16(L.d.k, L.d.stride, mb, grid, s, a);
  else rc = launch_conv_stem_bf16(L.d.k, L.d.stride, mb, grid, s, a);
  if (rc != CPRUNE_OK) return rc;
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

// The 16-bit 7x7 / stride 2 first-layer kernel on the caller's NCHW input, with or without the max-pool behind it.
static int net_run_stem7(cprune_net* net, int i, int n, const void* x, void* dst, hipStream_t s) {
  const NetLayer& L = net->layers[i];
  const bool pool = L.stem7 == 2;
  StemArgs a;
  a.x = x; a.w = L.w_stem7; a.bias = L.b; a.y = dst;
  a.N = n; a.C = L.d.c_in; a.H = L.h_in; a.W = L.w_in; a.Ho = L.h_out; a.Wo = L.w_out;
  a.O = L.d.c_out; a.Cop = L.cp_out; a.pad = L.d.pad; a.act = L.d.act;
  const int mb = L.d.c_out <= 32 ? 2 : 4;
  a.tiles_m = (a.O + mb * 16 - 1) / (mb * 16);
  if (pool) {
    const NetLayer& P = net->layers[L.pool3];
    a.y = P.act; a.Hp = P.h_out; a.Wp = P.w_out; a.Cop = P.cp_out;
    a.tiles_y = (a.Hp + 6) / 7; a.tiles_x = (a.Wp + 6) / 7;
  } else {
    a.tiles_y = (a.Ho + 15) / 16; a.tiles_x = (a.Wo + 15) / 16;
  }
  a.vec_out = (a.Cop % 4) == 0 ? 1 : 0;
  a.magic_x = a.tiles_x > 1 ? (unsigned)((0x100000000ull + a.tiles_x - 1) / a.tiles_x) : 0u;
  a.magic_y = a.tiles_y > 1 ? (unsigned)((0x100000000ull + a.tiles_y - 1) / a.tiles_y) : 0u;
  const long ptiles = (long)n * a.tiles_y * a.tiles_x;
  // as many workers as stay resident: weight tile + patch (+ the conv block the pool reads)
  const long lds = (long)mb * 16 * (kStem7K * 2 + 16) + 37L * 320 + (pool ? 256L * (mb * 32 + 16) : 16L);
  long per_cu = (160 * 1024) / lds;
  per_cu = per_cu > 8 ? 8 : (per_cu < 1 ? 1 : per_cu);
  const long workers = ptiles < 256 * per_cu ? ptiles : 256 * per_cu;
  dim3 grid((unsigned)workers, (unsigned)a.tiles_m);
  int rc;
  if (net->dtype == CPRUNE_F16) rc = launch_conv_stem7_f16(mb, pool ? 1 : 0, grid, s, a);
  else if (net->dtype == CPRUNE_BF16) rc = launch_conv_stem7_bf16(mb, pool ? 1 : 0, grid, s, a);
  else rc = CPRUNE_ERR_UNSUPPORTED;
  if (rc != CPRUNE_OK) return rc;
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

// First layer L.fuse_stem and the 3x3 layer i in one kernel: reads the caller's NCHW image.
static int net_run_stem2(cprune_net* net, int i, int n, const void* x, void* dst, hipStream_t s) {
  const NetLayer& L = net->layers[i];
  const NetLayer& F = net->layers[L.fuse_stem];
  const cprune_conv_desc d2 = layer_conv_desc(*net, L, n);
  return launch_conv_stem2(d2, layer_layout(L), x, F.d.c_in, F.w_stem, F.b, F.d.c_out, F.d.act, L.w, L.b, dst, s);
}

// Depthwise layer P.fuse_dw and the 1x1 layer i in one kernel: reads the depthwise layer's input.
static int net_run_dwproj(cprune_net* net, int i, int n, void* dst, hipStream_t s) {
  const NetLayer& P = net->layers[i];
  const NetLayer& D = net->layers[P.fuse_dw];
  const size_t es = dtype_size(net->dtype);
  DwProjArgs a;
  a.x = net->layers[D.d.input].act;
  a.wdw = D.w; a.bdw = D.b; a.wp = P.w; a.bp = P.b;
  a.res = P.d.residual >= 0 ? net->layers[P.d.residual].act : nullptr;
  a.y = dst;
  a.N = n; a.H = D.h_in; a.W = D.w_in; a.Ho = D.h_out; a.Wo = D.w_out;
  a.Ce = D.d.c_out; a.Cpe = D.cp_in; a.O = P.d.c_out; a.Cop = P.cp_out;
  a.pad = D.d.pad; a.act_dw = D.d.act; a.act_out = P.d.act;
  const int mb = P.d.c_out <= 32 ? 2 : (P.d.c_out <= 64 ? 4 : 8);
  a.tiles_y = (a.Ho + 7) / 8; a.tiles_x = (a.Wo + 7) / 8; a.tiles_m = (a.O + mb * 16 - 1) / (mb * 16);
  a.x_bytes = (unsigned)((size_t)n * a.H * a.W * a.Cpe * es);
  a.wp_bytes = (unsigned)((size_t)a.O * a.Cpe * es);
  a.wdw_bytes = (unsigned)((size_t)D.d.k * D.d.k * a.Cpe * es);
  a.vec_out = (a.Cop % 4) == 0 ? 1 : 0;
  dim3 grid((unsigned)(n * a.tiles_y * a.tiles_x * a.tiles_m));
  int rc;
  if (net->dtype == CPRUNE_F32) rc = launch_dwproj_f32(D.d.k, D.d.stride, mb, P.dw_ks, grid, s, a);
  else if (net->dtype == CPRUNE_F16) rc = launch_dwproj_f16(D.d.k, D.d.stride, mb, P.dw_ks, grid, s, a);
  else rc = launch_dwproj_bf16(D.d.k, D.d.stride, mb, P.dw_ks, grid, s, a);
  if (rc != CPRUNE_OK) return rc;
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

// Expansion P.fuse_block, depthwise P.fuse_dw and projection i in one kernel: reads the expansion's input.
static bool mbconv_fits(const cprune_net& net, const NetLayer& E, const NetLayer& D, const NetLayer& P, int* mb_out,
                        size_t* lds_out) {
  const int es = (int)dtype_size(net.dtype);
  if (P.d.c_out > 128) return false;
  const int mb = P.d.c_out <= 32 ? 2 : (P.d.c_out <= 64 ? 4 : 8);
  MbConvArgs lay;
  const size_t lds = mbconv_lds_layout(D.d.k, D.d.stride, mb, E.cp_in, D.cp_in, es, &lay);
  if (lds > 160 * 1024) return false;      // the block's weights do not fit beside its tiles
  const int ph = 7 * D.d.stride + D.d.k, npatchp = (ph * ph + 31) / 32 * 32;
  if ((long)npatchp * lay.xq > 256L * 10) return false;   // the next patch travels in ten registers per thread
  if (mb_out) *mb_out = mb;
  if (lds_out) *lds_out = lds;
  return true;
}

static int net_run_mbconv(cprune_net* net, int i, int n, void* dst, hipStream_t s) {
  const NetLayer& P = net->layers[i];
  const NetLayer& D = net->layers[P.fuse_dw];
  const NetLayer& E = net->layers[P.fuse_block];
  const size_t es = dtype_size(net->dtype);
  int mb = 0;
  size_t lds = 0;
  if (!mbconv_fits(*net, E, D, P, &mb, &lds)) return CPRUNE_ERR_UNSUPPORTED;
  MbConvArgs a;
  mbconv_lds_layout(D.d.k, D.d.stride, mb, E.cp_in, D.cp_in, (int)es, &a);
  a.x = net->layers[E.d.input].act;
  a.we = E.w; a.be = E.b; a.wdw = D.w; a.bdw = D.b; a.wp = P.w; a.bp = P.b;
  a.res = P.d.residual >= 0 ? net->layers[P.d.residual].act : nullptr;
  a.y = dst;
  a.N = n; a.H = D.h_in; a.W = D.w_in; a.Ho = D.h_out; a.Wo = D.w_out;
  a.Cpi = E.cp_in; a.Ce = D.d.c_out; a.Cpe = D.cp_in; a.O = P.d.c_out; a.Cop = P.cp_out;
  a.pad = D.d.pad; a.act_e = E.d.act; a.act_dw = D.d.act; a.act_out = P.d.act;
  a.tiles_y = (a.Ho + 7) / 8; a.tiles_x = (a.Wo + 7) / 8;
  a.x_bytes = (unsigned)((size_t)n * a.H * a.W * a.Cpi * es);
  a.we_bytes = (unsigned)((size_t)a.Ce * a.Cpi * es);
  a.wp_bytes = (unsigned)((size_t)a.O * a.Cpe * es);
  a.wdw_bytes = (unsigned)((size_t)D.d.k * D.d.k * a.Cpe * es);
  a.vec_out = (a.Cop % 4) == 0 ? 1 : 0;
  // as many work-groups as stay resident (LDS decides), each walking over its share of the pixel blocks
  const long ntiles = (long)n * a.tiles_y * a.tiles_x;
  long per_cu = (long)(160 * 1024 / lds);
  per_cu = per_cu > 4 ? 4 : (per_cu < 1 ? 1 : per_cu);
  const long workers = ntiles < 256 * per_cu ? ntiles : 256 * per_cu;
  dim3 grid((unsigned)workers);
  int rc;
  if (net->dtype == CPRUNE_F32) rc = launch_mbconv_f32(D.d.k, D.d.stride, mb, grid, lds, s, a);
  else if (net->dtype == CPRUNE_F16) rc = launch_mbconv_f16(D.d.k, D.d.stride, mb, grid, lds, s, a);
  else rc = launch_mbconv_bf16(D.d.k, D.d.stride, mb, grid, lds, s, a);
  if (rc != CPRUNE_OK) return rc;
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

static int net_run_layer(cprune_net* net, int i, int n, const void* x, void* out_override, hipStream_t s) {
  NetLayer& L = net->layers[i];
  const void* src = L.d.input < 0 ? (L.nchw_in ? x : net->x_cl) : net->layers[L.d.input].act;
  void* dst = out_override ? out_override : L.act;
  if (L.fused_away) return CPRUNE_OK;
  if (L.fuse_block >= 0) return net_run_mbconv(net, i, n, dst, s);
  if (L.fuse_dw >= 0) return net_run_dwproj(net, i, n, dst, s);
  if (L.fuse_stem >= 0) return net_run_stem2(net, i, n, x, dst, s);
  if (L.stem7) return net_run_stem7(net, i, n, src, dst, s);
  if (L.stem) return net_run_stem(net, i, n, src, dst, s);
  switch (L.d.kind) {
    case CPRUNE_LAYER_CONV:
    case CPRUNE_LAYER_FC: {
      cprune_conv_desc d = layer_conv_desc(*net, L, n);
      const ConvLayout lay = layer_layout(L);
      const void* res = L.d.residual >= 0 ? net->layers[L.d.residual].act : nullptr;
      int v = -1;
      if (d.groups == 1) v = (n == net->max_batch) ? L.variant : cached_or_heuristic_variant(d, nullptr, lay);
      return conv_dispatch(d, src, L.w, L.b, res, dst, v, net->ws, net->ws_bytes, s, lay);
    }
    case CPRUNE_LAYER_MAXPOOL:
      if (L.alias || L.in_producer) return CPRUNE_OK;
      return launch_maxpool_nhwc(src, n, L.cp_in, L.h_in, L.w_in, L.d.k, L.d.stride, L.d.pad, net->dtype, dst, s);
    case CPRUNE_LAYER_GAVGPOOL:
      return launch_gavgpool_nhwc(src, n, L.cp_in, L.h_in * L.w_in, net->dtype, dst, s);
  }
  return CPRUNE_ERR_INVALID_ARG;
}

// Device time of running the given layers one after the other, as they are configured right now:
// the faster of two timed passes of six repetitions each, after one untimed pass.  What the
// create-time choices between two forms of the same layers are decided by.
static int time_layers(cprune_net* net, const int* layers, int n_layers, int batch, const void* x, hipStream_t s,
                       float* ms_out) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  CPRUNE_HIP_TRY(hipEventCreate(&e0));
  hipError_t e = hipEventCreate(&e1);
  if (e != hipSuccess) { hipEventDestroy(e0); set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
  int rc = CPRUNE_OK;
  float best = 0.f;
  for (int pass = 0; pass < 3 && rc == CPRUNE_OK && e == hipSuccess; ++pass) {
    e = hipEventRecord(e0, s);
    for (int it = 0; it < 6 && rc == CPRUNE_OK; ++it)
      for (int k = 0; k < n_layers && rc == CPRUNE_OK; ++k) rc = net_run_layer(net, layers[k], batch, x, nullptr, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
    if (pass == 1 || (pass == 2 && t < best)) best = t;
  }
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  if (rc != CPRUNE_OK) return rc;
  if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
  *ms_out = best;
  return CPRUNE_OK;
}

// The last layer writes straight into the caller's buffer when its map is 1x1 (its
// channel stride is then the dense channel count); otherwise its buffer is converted.
static int net_enqueue(cprune_net* net, const void* x, int n, void* logits, hipStream_t s) {
  const int nl = (int)net->layers.size();
  int rc = CPRUNE_OK;
  if (net->convert_input) rc = launch_nchw_to_nhwc(x, n, net->in_c, net->in_h * net->in_w, net->in_cp, net->dtype, net->x_cl, s);
  if (rc != CPRUNE_OK) return rc;
  const NetLayer& last = net->layers[nl - 1];
  const bool direct = last.h_out * last.w_out == 1;
  for (int i = 0; i < nl; ++i) {
    rc = net_run_layer(net, i, n, x, (i == nl - 1 && direct) ? logits : nullptr, s);
    if (rc != CPRUNE_OK) return rc;
  }
  if (!direct)
    rc = launch_nhwc_to_nchw(last.act, n, last.d.c_out, last.h_out * last.w_out, last.cp_out, net->dtype, logits, s);
  return rc;
}

extern "C" int cprune_net_create(const cprune_layer_desc* layers, int n_layers, int in_c, int in_h,
                                 int in_w, int max_batch, cprune_dtype dtype, int tune, void* stream,
                                 cprune_net** out) {
  if (!layers || !out || n_layers < 1 || in_c < 1 || in_h < 1 || in_w < 1 || max_batch < 1) return CPRUNE_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return CPRUNE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  cprune_net* net = new cprune_net();
  net->in_c = in_c; net->in_h = in_h; net->in_w = in_w; net->max_batch = max_batch; net->dtype = dtype;
  net->in_cp = round_up_vec(in_c, dtype);
  net->layers.resize(n_layers);
  const size_t es = dtype_size(dtype);
  const long lim = 1L << 31;
  int rc = CPRUNE_OK;
  // shapes and validation
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& L = net->layers[i];
    L.d = layers[i];
    const cprune_layer_desc& d = L.d;
    if (d.input < -1 || d.input >= i || d.residual < -1 || d.residual >= i) { rc = CPRUNE_ERR_INVALID_ARG; break; }
    int c, h, w;
    if (d.input < 0) { c = in_c; h = in_h; w = in_w; L.cp_in = net->in_cp; }
    else { const NetLayer& S = net->layers[d.input]; c = S.d.c_out; h = S.h_out; w = S.w_out; L.cp_in = S.cp_out; }
    L.h_in = h; L.w_in = w;
    if (d.kind == CPRUNE_LAYER_FC) {
      if (d.c_in != c || d.c_out < 1 || !d.weight || !act_ok(d.act) || d.residual >= 0) { rc = CPRUNE_ERR_INVALID_ARG; break; }
      if (h > 7 || w > 7) { rc = CPRUNE_ERR_UNSUPPORTED; break; }
      L.h_out = L.w_out = 1;
    } else if (d.kind == CPRUNE_LAYER_GAVGPOOL) {
      if (d.c_in != c || d.c_out != c) { rc = CPRUNE_ERR_INVALID_ARG; break; }
      L.h_out = L.w_out = 1;
    } else if (d.kind == CPRUNE_LAYER_MAXPOOL || d.kind == CPRUNE_LAYER_CONV) {
      if (d.c_in != c || d.k < 1 || d.stride < 1 || d.pad < 0 || h + 2 * d.pad < d.k || w + 2 * d.pad < d.k) { rc = CPRUNE_ERR_INVALID_ARG; break; }
      L.h_out = conv_out_dim(h, d.k, d.stride, d.pad);
      L.w_out = conv_out_dim(w, d.k, d.stride, d.pad);
      if (d.kind == CPRUNE_LAYER_MAXPOOL) {
        if (d.c_out != c || d.pad >= d.k) { rc = CPRUNE_ERR_INVALID_ARG; break; }
      } else if (!d.weight) { rc = CPRUNE_ERR_INVALID_ARG; break; }
    } else { rc = CPRUNE_ERR_INVALID_ARG; break; }
    if (d.kind == CPRUNE_LAYER_CONV || d.kind == CPRUNE_LAYER_FC) {
      cprune_conv_desc cd = layer_conv_desc(*net, L, max_batch);
      rc = validate_conv_desc(&cd);
      if (rc != CPRUNE_OK) break;
    }
    // pools keep their input's stride; a final 1x1 map is written dense for the caller
    const bool last_dense = (i == n_layers - 1) && L.h_out * L.w_out == 1;
    if (d.kind == CPRUNE_LAYER_MAXPOOL || d.kind == CPRUNE_LAYER_GAVGPOOL) L.cp_out = L.cp_in;
    else L.cp_out = last_dense ? d.c_out : round_up_vec(d.c_out, dtype);
    if (last_dense && L.cp_out != d.c_out) { rc = CPRUNE_ERR_UNSUPPORTED; break; }  // a pool cannot end a net densely
    if (d.residual >= 0) {
      const NetLayer& R = net->layers[d.residual];
      if (d.kind != CPRUNE_LAYER_CONV || R.d.c_out != d.c_out || R.h_out != L.h_out || R.w_out != L.w_out ||
          R.cp_out != L.cp_out) { rc = CPRUNE_ERR_INVALID_ARG; break; }
    }
    L.per_image = (size_t)L.cp_out * L.h_out * L.w_out;
    if ((long)L.per_image * max_batch * (long)es >= lim || (long)L.cp_in * h * w * max_batch * (long)es >= lim) { rc = CPRUNE_ERR_UNSUPPORTED; break; }
  }
  if (rc != CPRUNE_OK) { net_free(net); return rc; }

  // A 3x3 / stride 1 / pad 1 conv on a 2x2 map reads the whole input map for every output pixel:
  // it runs as one matrix product per image, 4/9 of the multiply-adds of the nine-tap form
  // (the other 5/9 would multiply padding).
  for (int i = 0; i < n_layers; ++i) {
    NetLayer& L = net->layers[i];
    const cprune_layer_desc& d = L.d;
    if (d.kind == CPRUNE_LAYER_CONV && d.groups == 1 && d.k == 3 && d.stride == 1 && d.pad == 1 &&
        L.h_in == 2 && L.w_in == 2 && L.cp_out == round_up_vec(d.c_out, dtype))
      L.map2x2 = true;
  }

  // A 2x2 / stride 2 max-pool whose only producer is a plain 3x3 stride-1 conv that nobody
  // else reads runs in that conv's epilogue: one launch and one round trip through HBM less.
  for (int i = 0; i < n_layers; ++i) {
    NetLayer& Pl = net->layers[i];
    const cprune_layer_desc& pd = Pl.d;
    if (pd.kind != CPRUNE_LAYER_MAXPOOL || pd.k != 2 || pd.stride != 2 || pd.pad != 0 || pd.input < 0) continue;
    NetLayer& Cv = net->layers[pd.input];
    const cprune_layer_desc& cd = Cv.d;
    if (cd.kind != CPRUNE_LAYER_CONV || cd.groups != 1 || cd.k != 3 || cd.stride != 1 || cd.pad != 1 || cd.residual >= 0) continue;
    if ((Cv.h_out & 1) || (Cv.w_out & 1) || i == n_layers - 1) continue;
    bool shared = false;
    for (int j = 0; j < n_layers; ++j)
      if (j != i && (net->layers[j].d.input == pd.input || net->layers[j].d.residual == pd.input)) shared = true;
    if (shared) continue;
    // only where some variant can run the layer with the pool in its epilogue (none can on e.g. a 2 x 18 map)
    Cv.fused_pool = true;
    const cprune_conv_desc fd = layer_conv_desc(*net, Cv, max_batch);
    const ConvLayout fl = layer_layout(Cv);
    bool runnable = false;
    for (int v = 0; v < num_variants() && !runnable; ++v) runnable = variant_supports(fd, v, fl);
    if (!runnable) { Cv.fused_pool = false; continue; }
    Cv.per_image = (size_t)Cv.cp_out * Pl.h_out * Pl.w_out;
    Pl.alias = true;
  }

  // A dense conv on the network input reads the caller's NCHW tensor directly (its few input
  // channels gain nothing from the channels-last vector loads) and writes channels-last.
  net->convert_input = false;
  for (int i = 0; i < n_layers; ++i) {
    NetLayer& L = net->layers[i];
    if (L.d.input >= 0) continue;
    if (L.d.kind == CPRUNE_LAYER_CONV && L.d.groups == 1 && L.d.c_in <= 4 && !L.fused_pool && !L.map2x2 &&
        L.d.residual < 0 && L.cp_out == round_up_vec(L.d.c_out, dtype))
      L.nchw_in = true;
    else
      net->convert_input = true;
  }

  auto dev_alloc = [&](size_t bytes, void** p) -> int {
    hipError_t e = hipMalloc(p, bytes ? bytes : 16);
    if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
    net->allocs.push_back(*p);
    return CPRUNE_OK;
  };
  // weights (repacked channels-last), biases, activations, scratch
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& L = net->layers[i];
    const cprune_layer_desc& d = L.d;
    if (L.map2x2) {
      const int cpo = round_up_vec(d.c_out, dtype);
      const size_t nw = (size_t)16 * cpo * L.cp_in;
      if ((long)nw * (long)es >= lim) { rc = CPRUNE_ERR_UNSUPPORTED; break; }
      rc = dev_alloc(nw * es, &L.w);
      if (rc == CPRUNE_OK) rc = dev_alloc((size_t)4 * cpo * sizeof(float), (void**)&L.b);
      if (rc != CPRUNE_OK) break;
      rc = launch_repack_map2x2(d.weight, d.bias, d.c_out, d.c_in, L.cp_in, cpo, L.fused_pool ? 1 : 0, dtype, L.w, L.b, s);
      if (rc != CPRUNE_OK) break;
      cprune_conv_desc cd = layer_conv_desc(*net, L, max_batch);
      size_t need = conv_ws_bytes(cd, -1, layer_layout(L));
      if (need > net->ws_bytes) net->ws_bytes = need;
    } else if (L.nchw_in) {
      const size_t nw = (size_t)d.c_out * d.c_in * d.k * d.k;
      rc = dev_alloc(nw * es, &L.w);
      if (rc != CPRUNE_OK) break;
      hipError_t e = hipMemcpyAsync(L.w, d.weight, nw * es, hipMemcpyDeviceToDevice, s);
      if (e == hipSuccess && d.bias) {
        rc = dev_alloc((size_t)d.c_out * sizeof(float), (void**)&L.b);
        if (rc != CPRUNE_OK) break;
        e = hipMemcpyAsync(L.b, d.bias, (size_t)d.c_out * sizeof(float), hipMemcpyDeviceToDevice, s);
      }
      if (e != hipSuccess) { set_last_hip_error(e); rc = CPRUNE_ERR_DEVICE; break; }
      cprune_conv_desc cd = layer_conv_desc(*net, L, max_batch);
      size_t need = conv_ws_bytes(cd, -1, layer_layout(L));
      if (need > net->ws_bytes) net->ws_bytes = need;
    } else if (d.kind == CPRUNE_LAYER_CONV || d.kind == CPRUNE_LAYER_FC) {
      const int khw = d.kind == CPRUNE_LAYER_FC ? L.h_in * L.w_in : d.k * d.k;
      const bool dw = d.kind == CPRUNE_LAYER_CONV && d.groups != 1;
      const size_t nw = (size_t)(dw ? 1 : d.c_out) * khw * L.cp_in;
      if ((long)nw * (long)es >= lim) { rc = CPRUNE_ERR_UNSUPPORTED; break; }
      rc = dev_alloc(nw * es, &L.w);
      if (rc != CPRUNE_OK) break;
      rc = launch_repack_weights(d.weight, dw ? 1 : d.c_out, d.c_in, khw, L.cp_in, dtype, L.w, s);
      if (rc != CPRUNE_OK) break;
      if (d.bias) {
        rc = dev_alloc((size_t)d.c_out * sizeof(float), (void**)&L.b);
        if (rc != CPRUNE_OK) break;
        hipError_t e = hipMemcpyAsync(L.b, d.bias, (size_t)d.c_out * sizeof(float), hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) { set_last_hip_error(e); rc = CPRUNE_ERR_DEVICE; break; }
      }
      if (!dw) {
        cprune_conv_desc cd = layer_conv_desc(*net, L, max_batch);
        size_t need = conv_ws_bytes(cd, -1, layer_layout(L));
        if (need > net->ws_bytes) net->ws_bytes = need;
      }
    }
    if (L.alias) { L.act = net->layers[d.input].act; continue; }
    const size_t abytes = L.per_image * max_batch * es;
    rc = dev_alloc(abytes, &L.act);
    if (rc != CPRUNE_OK) break;
    hipError_t e = hipMemsetAsync(L.act, 0, abytes, s);
    if (e != hipSuccess) { set_last_hip_error(e); rc = CPRUNE_ERR_DEVICE; break; }
  }
  if (rc == CPRUNE_OK && net->ws_bytes) rc = dev_alloc(net->ws_bytes, &net->ws);
  if (rc == CPRUNE_OK) {
    size_t ib = (size_t)max_batch * net->in_cp * in_h * in_w * es;
    rc = dev_alloc(ib, &net->x_cl);
    if (rc == CPRUNE_OK) {
      hipError_t e = hipMemsetAsync(net->x_cl, 0, ib, s);
      if (e != hipSuccess) { set_last_hip_error(e); rc = CPRUNE_ERR_DEVICE; }
    }
  }
  // 3x3 layers on small maps: a second copy of the weights in the operand order of the kernel made for them
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& L = net->layers[i];
    const cprune_layer_desc& d = L.d;
    if (!(d.kind == CPRUNE_LAYER_CONV && d.groups == 1 && d.k == 3 && d.stride == 1 && d.pad == 1)) continue;
    if (L.map2x2 || L.nchw_in || L.h_in < 3 || L.w_in < 3 || L.h_in > 32 || L.w_in > 32) continue;
    if (wave_packed_bytes(d.c_out, L.cp_in, dtype) >= ((size_t)1 << 31)) continue;   // 31-bit offsets in the kernel
    rc = dev_alloc(wave_packed_bytes(d.c_out, L.cp_in, dtype), &L.w_wave);
    if (rc == CPRUNE_OK) rc = launch_repack_wave(L.w, d.c_out, L.cp_in, dtype, L.w_wave, s);
  }
  // layers the reduction-split kernel can run (1x1 / stride 1, fully connected, 2x2 maps as one matrix; few
  // pixels): likewise a copy in its operand order
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& L = net->layers[i];
    if (!(L.d.kind == CPRUNE_LAYER_FC || (L.d.kind == CPRUNE_LAYER_CONV && L.d.groups == 1)) || L.nchw_in) continue;
    const cprune_conv_desc cd = layer_conv_desc(*net, L, max_batch);
    const ConvLayout lay = layer_layout(L);
    bool any = false;
    for (int v = 0; v < num_variants() && !any; ++v) any = variant(v).sched == -2 && variant_supports(cd, v, lay);
    if (!any) continue;
    const int k = lay.cp_in * cd.kh * cd.kw;
    if (rows_packed_bytes(cd.c_out, k, dtype) >= ((size_t)1 << 31)) continue;   // the kernel then reads the row layout
    rc = dev_alloc(rows_packed_bytes(cd.c_out, k, dtype), &L.w_rows);
    if (rc == CPRUNE_OK) rc = launch_repack_rows(L.w, cd.c_out, k, dtype, L.w_rows, s);
  }
  // variant per dense layer
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& L = net->layers[i];
    if (!(L.d.kind == CPRUNE_LAYER_FC || (L.d.kind == CPRUNE_LAYER_CONV && L.d.groups == 1))) continue;
    cprune_conv_desc cd = layer_conv_desc(*net, L, max_batch);
    const ConvLayout lay = layer_layout(L);
    bool timed = false;
    int v = cached_or_heuristic_variant(cd, &timed, lay);
    if (tune && !timed) {
      const void* src = L.d.input < 0 ? net->x_cl : net->layers[L.d.input].act;
      const void* res = L.d.residual >= 0 ? net->layers[L.d.residual].act : nullptr;
      rc = select_tile_impl(cd, src, L.w, L.b, res, L.act, net->ws, net->ws_bytes, 2, 6, &v, nullptr, nullptr, s, lay);
    }
    L.variant = v;
  }
  // A first layer with an image-like input (<= 3 channels; 3x3 or 7x7 window) has a kernel of its
  // own that keeps the whole reduction in LDS; with tune != 0 it is timed against the chosen variant
  // of the general kernel, otherwise it is taken.
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& L = net->layers[i];
    const cprune_layer_desc& d = L.d;
    if (!L.nchw_in || d.c_in > 3 || d.pad != d.k / 2) continue;
    if (!((d.k == 3 && (d.stride == 1 || d.stride == 2)) || (d.k == 7 && d.stride == 2))) continue;
    L.stem_ok = 1;
    {
      const int mb = d.c_out <= 32 ? 2 : 4;
      const int rows = (d.c_out + mb * 16 - 1) / (mb * 16) * (mb * 16);
      const int kp = stem_packed_k(d.k, dtype);
      rc = dev_alloc((size_t)rows * kp * es, &L.w_stem);
      if (rc == CPRUNE_OK) rc = launch_repack_stem(L.w, d.c_out, d.c_in * d.k * d.k, rows, kp, dtype, L.w_stem, s);
      if (rc != CPRUNE_OK) break;
    }
    bool use = true;
    if (tune) {
      float ms[2] = {0.f, 0.f};
      for (int form = 0; form < 2 && rc == CPRUNE_OK; ++form) {   // 0: general kernel, 1: first-layer kernel
        L.stem = form == 1;
        rc = time_layers(net, &i, 1, max_batch, net->x_cl, s, &ms[form]);
      }
      use = ms[1] < ms[0];
    }
    L.stem = use;
    if (use) L.variant = -1;
  }

  // 16-bit data, 7x7 / stride 2 / pad 3 on the image (the first layer of the ImageNet networks): a kernel whose
  // reduction order makes every MFMA operand one LDS read, and which can run the 3x3 / stride 2 / pad 1 max-pool
  // behind the layer as well when nobody else reads the conv map.  With tune != 0 the three forms (as decided so far;
  // that kernel; that kernel with the pool) are timed and the fastest kept; otherwise the most fused one is taken.
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& L = net->layers[i];
    const cprune_layer_desc& d = L.d;
    if (dtype == CPRUNE_F32 || !L.nchw_in || d.c_in > 3 || d.k != 7 || d.stride != 2 || d.pad != 3 || d.residual >= 0) continue;
    {
      const int mb = d.c_out <= 32 ? 2 : 4;
      const int rows = (d.c_out + mb * 16 - 1) / (mb * 16) * (mb * 16);
      rc = dev_alloc((size_t)rows * kStem7K * es, &L.w_stem7);
      if (rc == CPRUNE_OK) rc = launch_repack_stem7(L.w, d.c_out, d.c_in, rows, dtype, L.w_stem7, s);
      if (rc != CPRUNE_OK) break;
    }
    int reader = -1, readers = 0;
    for (int j = 0; j < n_layers; ++j) {
      if (net->layers[j].d.input == i) { reader = j; ++readers; }
      if (net->layers[j].d.residual == i) readers += 2;
    }
    if (readers == 1 && reader != n_layers - 1) {
      const cprune_layer_desc& pd = net->layers[reader].d;
      if (pd.kind == CPRUNE_LAYER_MAXPOOL && pd.k == 3 && pd.stride == 2 && pd.pad == 1) L.pool3 = reader;
    }
    auto set_form = [&](int form) {
      L.stem7 = form;
      if (L.pool3 >= 0) net->layers[L.pool3].in_producer = form == 2;
    };
    const int n_forms = L.pool3 >= 0 ? 3 : 2;
    int best = n_forms - 1;
    if (tune) {
      const int pair[2] = {i, L.pool3};
      float ms[3] = {0.f, 0.f, 0.f};
      for (int form = 0; form < n_forms && rc == CPRUNE_OK; ++form) {
        set_form(form);
        rc = time_layers(net, pair, L.pool3 >= 0 ? 2 : 1, max_batch, net->x_cl, s, &ms[form]);
      }
      best = 0;
      for (int form = 1; form < n_forms; ++form)
        if (ms[form] < ms[best]) best = form;
    }
    set_form(best);
    if (best) L.variant = -1;
  }

  // A first layer (3x3 / stride 1, at most 32 filters) whose only reader is another 3x3 / stride 1 conv can run
  // inside that conv's kernel: the largest activation of a VGG-style network is then never written.  With
  // tune != 0 both forms are timed and the faster kept; otherwise only cprune_net_fuse_first_layers turns it on.
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& F = net->layers[i];
    if (!(F.stem_ok && F.nchw_in && F.d.k == 3 && F.d.stride == 1 && F.d.pad == 1 && F.d.residual < 0 && !F.fused_pool)) continue;
    int reader = -1, readers = 0;
    for (int j = 0; j < n_layers; ++j) {
      if (net->layers[j].d.input == i) { reader = j; ++readers; }
      if (net->layers[j].d.residual == i) readers += 2;
    }
    if (readers != 1 || i == n_layers - 1) continue;
    NetLayer& L = net->layers[reader];
    if (!(L.d.kind == CPRUNE_LAYER_CONV && L.d.groups == 1 && L.d.residual < 0 && !L.map2x2 && !L.nchw_in)) continue;
    if (!conv_stem2_supported(layer_conv_desc(*net, L, max_batch), layer_layout(L), F.d.c_in, F.d.c_out)) continue;
    F.stem_reader = reader;
    bool fuse = false;
    if (tune) {
      const int pair[2] = {i, reader};
      float ms[2] = {0.f, 0.f};
      for (int form = 0; form < 2 && rc == CPRUNE_OK; ++form) {   // 0: layers apart as decided so far, 1: one kernel
        F.fused_away = form == 1;
        L.fuse_stem = form == 1 ? i : -1;
        rc = time_layers(net, pair, 2, max_batch, net->x_cl, s, &ms[form]);
      }
      fuse = ms[1] < ms[0];
    }
    F.fused_away = fuse;
    L.fuse_stem = fuse ? i : -1;
    if (fuse) L.variant = -1;
  }

  // A depthwise conv whose only reader is a 1x1 conv can run inside that conv's kernel: the
  // expanded activations are then read once and never written.  It pays on large maps (enough
  // 8x8 pixel blocks to fill the chip); with tune != 0 both forms are timed and the faster kept.
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& D = net->layers[i];
    const cprune_layer_desc& dd = D.d;
    if (!(dd.kind == CPRUNE_LAYER_CONV && dd.groups != 1 && dd.input >= 0 && dd.residual < 0)) continue;
    if (!((dd.k == 3 || dd.k == 5) && (dd.stride == 1 || dd.stride == 2) && dd.pad == dd.k / 2)) continue;
    int reader = -1, readers = 0;
    for (int j = 0; j < n_layers; ++j) {
      if (net->layers[j].d.input == i) { reader = j; ++readers; }
      if (net->layers[j].d.residual == i) readers += 2;
    }
    if (readers != 1 || i == n_layers - 1) continue;
    NetLayer& P = net->layers[reader];
    const cprune_layer_desc& pd = P.d;
    if (!(pd.kind == CPRUNE_LAYER_CONV && pd.groups == 1 && pd.k == 1 && pd.stride == 1 && pd.pad == 0)) continue;
    if (P.cp_out != round_up_vec(pd.c_out, dtype) || P.nchw_in || P.map2x2 || P.fused_pool) continue;
    D.dw_reader = reader;
    const int mt = pd.c_out <= 32 ? 32 : (pd.c_out <= 64 ? 64 : 128);
    const long groups = (long)max_batch * ((D.h_out + 7) / 8) * ((D.w_out + 7) / 8) * ((pd.c_out + mt - 1) / mt);
    // Few pixel blocks (small maps) leave one group of four wavefronts per compute unit, whose channel
    // loop is a chain of waits: then 2 or 4 groups share a block and split the channel chunks.
    const int ks_max = (dd.k == 3 && dd.stride == 1) ? 4 : 2;
    P.dw_ks = groups <= 320 ? ks_max : (groups <= 640 ? 2 : 1);
    bool fuse = groups >= 512;
    if (tune) {
      const int pair[2] = {i, reader};
      float apart = 0.f, best = 0.f;
      D.fused_away = false; P.fuse_dw = -1;
      rc = time_layers(net, pair, 2, max_batch, nullptr, s, &apart);
      D.fused_away = true; P.fuse_dw = i;
      int best_ks = 1;
      for (int ks = 1; ks <= ks_max && rc == CPRUNE_OK; ks *= 2) {
        float ms = 0.f;
        P.dw_ks = ks;
        rc = time_layers(net, pair, 2, max_batch, nullptr, s, &ms);
        if (ks == 1 || ms < best) { best = ms; best_ks = ks; }
      }
      P.dw_ks = best_ks;
      fuse = best < apart;
    }
    D.fused_away = fuse;
    P.fuse_dw = fuse ? i : -1;
    if (fuse) P.variant = -1;
  }
  // When the depthwise layer's input is a 1x1 expansion that nobody else reads, the whole
  // inverted-residual block can be one kernel, and the expanded activations never reach memory.
  // It needs the projection's filters in one tile (at most 128) and all weights of the three layers
  // in LDS beside the tiles; with tune != 0 it is timed against the layers as decided so far and
  // taken when faster, otherwise only cprune_net_fuse_block turns it on.
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    NetLayer& D = net->layers[i];
    if (D.dw_reader < 0 || D.d.input < 0) continue;
    NetLayer& E = net->layers[D.d.input];
    NetLayer& P = net->layers[D.dw_reader];
    const cprune_layer_desc& ed = E.d;
    if (!(ed.kind == CPRUNE_LAYER_CONV && ed.groups == 1 && ed.k == 1 && ed.stride == 1 && ed.pad == 0)) continue;
    if (ed.input < 0 || ed.residual >= 0 || E.nchw_in || E.map2x2 || E.fused_pool || E.fuse_dw >= 0) continue;
    if (E.cp_out != round_up_vec(ed.c_out, dtype) || E.cp_out != D.cp_in) continue;
    int readers = 0;
    for (int j = 0; j < n_layers; ++j) {
      if (net->layers[j].d.input == D.d.input) ++readers;
      if (net->layers[j].d.residual == D.d.input) readers += 2;
    }
    if (readers != 1 || !mbconv_fits(*net, E, D, P, nullptr, nullptr)) continue;
    D.block_expand = D.d.input;
    bool fuse = false;   // untimed, the layers stay apart: so far the one-kernel form has not been the faster one
    const bool dw_fused = D.fused_away;
    if (tune) {
      float ms[2] = {0.f, 0.f};
      const int block[3] = {D.d.input, i, D.dw_reader};
      for (int form = 0; form < 2 && rc == CPRUNE_OK; ++form) {   // 0: as decided so far, 1: one kernel
        E.fused_away = form == 1;
        D.fused_away = form == 1 || dw_fused;
        P.fuse_dw = D.fused_away ? i : -1;
        P.fuse_block = form == 1 ? D.d.input : -1;
        rc = time_layers(net, block, 3, max_batch, nullptr, s, &ms[form]);
      }
      fuse = ms[1] < ms[0];
    }
    E.fused_away = fuse;
    D.fused_away = fuse || dw_fused;
    P.fuse_dw = D.fused_away ? i : -1;
    P.fuse_block = fuse ? D.d.input : -1;
    if (fuse) { P.variant = -1; E.variant = -1; }
  }
  if (rc == CPRUNE_OK) {
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) { set_last_hip_error(e); rc = CPRUNE_ERR_DEVICE; }
  }
  if (rc != CPRUNE_OK) { net_free(net); return rc; }
  *out = net;
  return CPRUNE_OK;
}

extern "C" int cprune_net_forward(cprune_net* net, const void* x, int n, void* logits, int use_graph,
                                  void* stream) {
  if (!net || !x || !logits) return CPRUNE_ERR_INVALID_ARG;
  if (n < 1 || n > net->max_batch) return CPRUNE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  net->last_n = n;
  if (!use_graph) return net_enqueue(net, x, n, logits, s);
  GraphKey key{n, x, logits};
  auto it = net->graphs.find(key);
  if (it == net->graphs.end()) {
    if (!net->capture_stream) CPRUNE_HIP_TRY(hipStreamCreateWithFlags(&net->capture_stream, hipStreamNonBlocking));
    hipStream_t cs = net->capture_stream;
    hipGraph_t graph = nullptr;
    CPRUNE_HIP_TRY(hipStreamBeginCapture(cs, hipStreamCaptureModeRelaxed));
    int rc = net_enqueue(net, x, n, logits, cs);
    hipError_t e = hipStreamEndCapture(cs, &graph);
    if (rc != CPRUNE_OK) { if (graph) hipGraphDestroy(graph); return rc; }
    if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    hipGraphDestroy(graph);
    if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
    if (net->graphs.size() >= kMaxGraphs) {
      // make room: the least recently replayed graph goes, once nothing can still be running it
      auto victim = net->graphs.begin();
      for (auto g = net->graphs.begin(); g != net->graphs.end(); ++g)
        if (g->second.last_use < victim->second.last_use) victim = g;
      hipError_t se = hipDeviceSynchronize();
      hipGraphExecDestroy(victim->second.exec);
      net->graphs.erase(victim);
      if (se != hipSuccess) { hipGraphExecDestroy(exec); set_last_hip_error(se); return CPRUNE_ERR_DEVICE; }
    }
    it = net->graphs.emplace(key, cprune_net::GraphEntry{exec, 0}).first;
  }
  it->second.last_use = ++net->graph_clock;
  CPRUNE_HIP_TRY(hipGraphLaunch(it->second.exec, s));
  return CPRUNE_OK;
}

extern "C" int cprune_net_layer_times(cprune_net* net, const void* x, int n, int iters, float* ms_out,
                                      void* stream) {
  if (!net || !x || !ms_out || iters < 1) return CPRUNE_ERR_INVALID_ARG;
  if (n < 1 || n > net->max_batch) return CPRUNE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int nl = (int)net->layers.size();
  hipEvent_t e0 = nullptr, e1 = nullptr;
  CPRUNE_HIP_TRY(hipEventCreate(&e0));
  hipError_t ec = hipEventCreate(&e1);
  if (ec != hipSuccess) { hipEventDestroy(e0); set_last_hip_error(ec); return CPRUNE_ERR_DEVICE; }
  net->last_n = n;
  int rc = CPRUNE_OK;
  if (net->convert_input) rc = launch_nchw_to_nhwc(x, n, net->in_c, net->in_h * net->in_w, net->in_cp, net->dtype, net->x_cl, s);
  // layer by layer, in order (so every layer finds its inputs): `iters` launches back to
  // back between two events, which is how the layer runs inside a forward pass
  for (int i = 0; i < nl && rc == CPRUNE_OK; ++i) {
    ms_out[i] = 0.0f;
    rc = net_run_layer(net, i, n, x, nullptr, s);   // untimed first run
    if (rc != CPRUNE_OK || net->layers[i].alias || net->layers[i].fused_away || net->layers[i].in_producer) continue;
    hipError_t e = hipEventRecord(e0, s);
    for (int it = 0; it < iters && rc == CPRUNE_OK && e == hipSuccess; ++it) rc = net_run_layer(net, i, n, x, nullptr, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e != hipSuccess) { set_last_hip_error(e); rc = CPRUNE_ERR_DEVICE; break; }
    ms_out[i] = ms / (float)iters;
  }
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  return rc;
}

extern "C" int cprune_net_copy_activation(cprune_net* net, int layer, int n, void* dst, size_t dst_bytes,
                                          void* stream) {
  if (!net || !dst || layer < 0 || layer >= (int)net->layers.size()) return CPRUNE_ERR_INVALID_ARG;
  if (n < 1 || n > net->max_batch) return CPRUNE_ERR_INVALID_ARG;
  const NetLayer& L = net->layers[layer];
  if (L.fused_pool || L.stem7 == 2) return CPRUNE_ERR_UNSUPPORTED;  // only the pooled map exists: ask for the pool layer
  if (L.fused_away) return CPRUNE_ERR_UNSUPPORTED;  // computed inside its consumer's kernel, never stored
  const size_t bytes = (size_t)L.d.c_out * L.h_out * L.w_out * n * dtype_size(net->dtype);
  if (dst_bytes < bytes) return CPRUNE_ERR_INVALID_ARG;
  return launch_nhwc_to_nchw(L.act, n, L.d.c_out, L.h_out * L.w_out, L.cp_out, net->dtype, dst, (hipStream_t)stream);
}

extern "C" int cprune_net_output_shape(const cprune_net* net, int* c_out, int* h_out, int* w_out) {
  if (!net || !c_out || !h_out || !w_out) return CPRUNE_ERR_INVALID_ARG;
  const NetLayer& L = net->layers.back();
  *c_out = L.d.c_out; *h_out = L.h_out; *w_out = L.w_out;
  return CPRUNE_OK;
}

extern "C" int cprune_net_layer_variant(const cprune_net* net, int layer, int* variant_out) {
  if (!net || !variant_out || layer < 0 || layer >= (int)net->layers.size()) return CPRUNE_ERR_INVALID_ARG;
  *variant_out = net->layers[layer].variant;
  return CPRUNE_OK;
}

extern "C" int cprune_net_task_table(const cprune_net* net, int* task_of_layer, int* n_tasks_out) {
  if (!net || !task_of_layer || !n_tasks_out) return CPRUNE_ERR_INVALID_ARG;
  std::map<DescKey, int> ids;
  for (size_t i = 0; i < net->layers.size(); ++i) {
    const NetLayer& L = net->layers[i];
    if (!(L.d.kind == CPRUNE_LAYER_FC || (L.d.kind == CPRUNE_LAYER_CONV && L.d.groups == 1))) { task_of_layer[i] = -1; continue; }
    const DescKey key = key_of(layer_conv_desc(*net, L, net->max_batch), layer_layout(L));
    auto it = ids.find(key);
    if (it == ids.end()) it = ids.emplace(key, (int)ids.size()).first;
    task_of_layer[i] = it->second;
  }
  *n_tasks_out = (int)ids.size();
  return CPRUNE_OK;
}

extern "C" int cprune_net_task_key(const cprune_net* net, int layer, int32_t* key_out) {
  if (!net || !key_out || layer < 0 || layer >= (int)net->layers.size()) return CPRUNE_ERR_INVALID_ARG;
  const NetLayer& L = net->layers[layer];
  if (!(L.d.kind == CPRUNE_LAYER_FC || (L.d.kind == CPRUNE_LAYER_CONV && L.d.groups == 1))) return CPRUNE_ERR_INVALID_ARG;
  const DescKey key = key_of(layer_conv_desc(*net, L, net->max_batch), layer_layout(L));
  static_assert(std::tuple_size<DescKey>::value == CPRUNE_TASK_KEY_INTS, "key length is part of the ABI");
  for (size_t i = 0; i < key.size(); ++i) key_out[i] = key[i];
  return CPRUNE_OK;
}

static void restore_variant(cprune_net* net, NetLayer& L) {
  if (L.variant < 0 && !L.stem && !L.stem7)
    L.variant = cached_or_heuristic_variant(layer_conv_desc(*net, L, net->max_batch), nullptr, layer_layout(L));
}

extern "C" int cprune_net_fuse_first_layers(cprune_net* net, int enable) {
  if (!net) return CPRUNE_ERR_INVALID_ARG;
  int first = -1;
  for (int i = 0; i < (int)net->layers.size(); ++i)
    if (net->layers[i].stem_reader >= 0) { first = i; break; }
  if (first < 0) return CPRUNE_ERR_UNSUPPORTED;
  CPRUNE_HIP_TRY(hipDeviceSynchronize());
  drop_graphs(net);
  NetLayer& F = net->layers[first];
  NetLayer& L = net->layers[F.stem_reader];
  F.fused_away = enable != 0;
  L.fuse_stem = enable ? first : -1;
  if (enable) L.variant = -1;
  else restore_variant(net, L);
  return CPRUNE_OK;
}

extern "C" int cprune_net_first_layer_form(cprune_net* net, int form) {
  if (!net || form < 0 || form > 2) return CPRUNE_ERR_INVALID_ARG;
  int first = -1;
  for (int i = 0; i < (int)net->layers.size(); ++i)
    if (net->layers[i].w_stem7) { first = i; break; }
  if (first < 0) return CPRUNE_ERR_UNSUPPORTED;
  NetLayer& L = net->layers[first];
  if (form == 2 && L.pool3 < 0) return CPRUNE_ERR_UNSUPPORTED;
  CPRUNE_HIP_TRY(hipDeviceSynchronize());
  drop_graphs(net);
  L.stem7 = form;
  if (L.pool3 >= 0) net->layers[L.pool3].in_producer = form == 2;
  if (form) L.variant = -1;
  else restore_variant(net, L);
  return CPRUNE_OK;
}

extern "C" int cprune_net_fuse_depthwise(cprune_net* net, int layer, int enable) {
  if (!net || layer < 0 || layer >= (int)net->layers.size()) return CPRUNE_ERR_INVALID_ARG;
  NetLayer& D = net->layers[layer];
  if (D.dw_reader < 0) return CPRUNE_ERR_UNSUPPORTED;
  CPRUNE_HIP_TRY(hipDeviceSynchronize());
  drop_graphs(net);
  NetLayer& P = net->layers[D.dw_reader];
  if (P.fuse_block >= 0) {             // leaves the one-kernel block form either way
    NetLayer& E = net->layers[P.fuse_block];
    E.fused_away = false;
    restore_variant(net, E);
    P.fuse_block = -1;
  }
  D.fused_away = enable != 0;
  P.fuse_dw = enable ? layer : -1;
  if (enable) P.variant = -1;
  else restore_variant(net, P);
  return CPRUNE_OK;
}

extern "C" int cprune_net_fuse_block(cprune_net* net, int layer, int enable) {
  if (!net || layer < 0 || layer >= (int)net->layers.size()) return CPRUNE_ERR_INVALID_ARG;
  NetLayer& D = net->layers[layer];
  if (D.dw_reader < 0 || D.block_expand < 0) return CPRUNE_ERR_UNSUPPORTED;
  CPRUNE_HIP_TRY(hipDeviceSynchronize());
  drop_graphs(net);
  NetLayer& P = net->layers[D.dw_reader];
  NetLayer& E = net->layers[D.block_expand];
  if (enable) {
    E.fused_away = true; D.fused_away = true;
    P.fuse_dw = layer; P.fuse_block = D.block_expand;
    P.variant = -1; E.variant = -1;
  } else if (P.fuse_block >= 0) {      // back to the depthwise + projection pair in one kernel, expansion on its own
    E.fused_away = false;
    restore_variant(net, E);
    P.fuse_block = -1;
  }
  return CPRUNE_OK;
}

extern "C" int cprune_net_layer_fused(const cprune_net* net, int layer, int* fused_out) {
  if (!net || !fused_out || layer < 0 || layer >= (int)net->layers.size()) return CPRUNE_ERR_INVALID_ARG;
  *fused_out = net->layers[layer].fused_away ? 1 : 0;
  return CPRUNE_OK;
}

extern "C" int cprune_net_set_layer_variant(cprune_net* net, int layer, int variant) {
  if (!net || layer < 0 || layer >= (int)net->layers.size()) return CPRUNE_ERR_INVALID_ARG;
  NetLayer& L = net->layers[layer];
  if (!(L.d.kind == CPRUNE_LAYER_FC || (L.d.kind == CPRUNE_LAYER_CONV && L.d.groups == 1))) return CPRUNE_ERR_INVALID_ARG;
  if (L.fuse_dw >= 0 || L.fuse_stem >= 0 || L.fused_away) return CPRUNE_ERR_INVALID_ARG;   // runs inside a fused kernel: no variants
  if (L.stem) L.stem = false;                          // a pinned variant means the general kernel
  if (L.stem7) {
    if (L.pool3 >= 0) net->layers[L.pool3].in_producer = false;
    L.stem7 = 0;
  }
  const cprune_conv_desc cd = layer_conv_desc(*net, L, net->max_batch);
  const ConvLayout lay = layer_layout(L);
  if (!variant_supports(cd, variant, lay)) return CPRUNE_ERR_UNSUPPORTED;
  if (conv_ws_bytes(cd, variant, lay) > net->ws_bytes) return CPRUNE_ERR_WORKSPACE;
  CPRUNE_HIP_TRY(hipDeviceSynchronize());
  drop_graphs(net);
  L.variant = variant;
  return CPRUNE_OK;
}

extern "C" int cprune_net_destroy(cprune_net* net) {
  if (!net) return CPRUNE_ERR_INVALID_ARG;
  hipError_t e = hipDeviceSynchronize();
  net_free(net);
  if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
  return CPRUNE_OK;
}
