// Filter ranking and channel gather (paper Section 3.5, last paragraph, and
// Section 2.1): L1 score per filter, rank by (score descending, index
// ascending), ascending kept list, weight gather with batch-norm folding,
// activation channel gather.  All bandwidth- or latency-bound; none of it is a
// contraction, so none of it uses the matrix cores.
//
// Two forms of the same kernels: one call per layer (cprune_rank_filters,
// cprune_gather_pruned_weights) and a plan over a whole network
// (cprune_prune_plan_*) that scores every ranked layer in one launch, ranks
// every layer in a second and gathers + folds every layer in a third.
#include "common.hpp"

#include <algorithm>
#include <mutex>
#include <vector>

namespace cprune {
namespace {

constexpr int kMaxRankFilters = 4096;
constexpr int kRowLds = 12288;          // floats of a source row the gather kernel stages in LDS
constexpr long kWaveFilterMax = 16384;  // longer filters are summed by a whole work-group

// ---- L1 score ------------------------------------------------------------------
// A lane's share of sum |f[i]|, i in [0, n): strided over `lanes` lanes in 16-byte pieces
// where the filter starts on a 16-byte boundary and n is a multiple of 4, element by
// element otherwise.  fp64 accumulation in index order per lane.
__device__ __forceinline__ double l1_lane_sum(const float* __restrict__ f, long n, int lane, int lanes) {
  double s = 0.0;
  if (((n & 3) == 0) && ((reinterpret_cast<uintptr_t>(f) & 15) == 0)) {
    const float4* f4 = reinterpret_cast<const float4*>(f);
    const long n4 = n >> 2;
    long i = lane;
    for (; i + 3L * lanes < n4; i += 4L * lanes) {   // four loads in flight per lane
      const float4 a = f4[i], b = f4[i + lanes], c = f4[i + 2L * lanes], d = f4[i + 3L * lanes];
      s += (double)fabsf(a.x); s += (double)fabsf(a.y); s += (double)fabsf(a.z); s += (double)fabsf(a.w);
      s += (double)fabsf(b.x); s += (double)fabsf(b.y); s += (double)fabsf(b.z); s += (double)fabsf(b.w);
      s += (double)fabsf(c.x); s += (double)fabsf(c.y); s += (double)fabsf(c.z); s += (double)fabsf(c.w);
      s += (double)fabsf(d.x); s += (double)fabsf(d.y); s += (double)fabsf(d.z); s += (double)fabsf(d.w);
    }
    for (; i < n4; i += lanes) {
      const float4 a = f4[i];
      s += (double)fabsf(a.x); s += (double)fabsf(a.y); s += (double)fabsf(a.z); s += (double)fabsf(a.w);
    }
  } else {
    for (long i = lane; i < n; i += lanes) s += (double)fabsf(f[i]);
  }
  return s;
}

// Sum over the 64 lanes of a wavefront in a fixed tree; every lane returns lane 0's total only in lane 0.
__device__ __forceinline__ double wave_sum(double s) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
  return s;
}

// Short filters: one wavefront per filter, four filters per work-group.  The order of
// additions depends only on the filter length and its alignment, so a score is
// reproducible bit for bit.  accumulate != 0: the sum is added to the score already there.
__global__ __launch_bounds__(256) void l1_score_wave_kernel(const float* __restrict__ w, long per_filter,
                                                            int c_out, double* __restrict__ scores,
                                                            int accumulate) {
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= c_out) return;
  const double s = wave_sum(l1_lane_sum(w + (long)j * per_filter, per_filter, threadIdx.x & 63, 64));
  if ((threadIdx.x & 63) == 0) scores[j] = accumulate ? scores[j] + s : s;
}

// Long filters: one work-group per filter (wavefront shuffles, then 4 partials in LDS).
__global__ __launch_bounds__(256) void l1_score_group_kernel(const float* __restrict__ w, long per_filter,
                                                             double* __restrict__ scores, int accumulate) {
  double s = wave_sum(l1_lane_sum(w + (long)blockIdx.x * per_filter, per_filter, threadIdx.x, 256));
  __shared__ double part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const double sum = (part[0] + part[1]) + (part[2] + part[3]);
    scores[blockIdx.x] = accumulate ? scores[blockIdx.x] + sum : sum;
  }
}

// ---- rank / select ---------------------------------------------------------------
// One work-group sorts a layer's filters by (score descending, index ascending) with a bitonic
// network in LDS (a total order: equal scores rank the lower index first, so the result is
// unique), then marks the first `keep` of that order as surviving and writes them out in
// ascending index: a filter's slot is the number of surviving filters with a lower index
// (wavefront ballots + a scan over the 16 wavefront totals).  The list is padded to a power of
// two with entries that rank behind every filter.
__device__ __forceinline__ bool ranks_before(double sa, int ia, double sb, int ib) {
  return sa > sb || (sa == sb && ia < ib);
}

__device__ __forceinline__ void rank_select(const double* __restrict__ scores, int c, int keep,
                                            int32_t* __restrict__ order, int32_t* __restrict__ kept,
                                            double* s, int* idx, unsigned char* alive, int* wave_total) {
  int n = 64;
  while (n < c) n <<= 1;
  for (int i = threadIdx.x; i < n; i += 1024) {
    s[i] = i < c ? scores[i] : -1.0;   // scores are sums of absolute values: never negative
    idx[i] = i;
  }
  __syncthreads();
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = threadIdx.x; t < (n >> 1); t += 1024) {
        const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;   // the pair this thread orders
        const bool up = (lo & k) == 0;                                       // direction of its subsequence
        const double sl = s[lo], sh = s[hi];
        const int il = idx[lo], ih = idx[hi];
        if (ranks_before(sh, ih, sl, il) == up) { s[lo] = sh; s[hi] = sl; idx[lo] = ih; idx[hi] = il; }
      }
      __syncthreads();
    }
  }
  for (int i = threadIdx.x; i < c; i += 1024) alive[i] = 0;
  __syncthreads();
  for (int rnk = threadIdx.x; rnk < c; rnk += 1024) {
    const int i = idx[rnk];
    if (order) order[rnk] = i;
    if (rnk < keep) alive[i] = 1;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int base = 0;   // surviving filters below the current round of 1024 indices
  for (int i0 = 0; i0 < c; i0 += 1024) {
    const int i = i0 + threadIdx.x;
    const bool live = i < c && alive[i];
    const unsigned long long mask = __ballot(live);
    if (lane == 0) wave_total[wave] = __popcll(mask);
    __syncthreads();
    int before = base;
    for (int k = 0; k < wave; ++k) before += wave_total[k];
    if (live) kept[before + __popcll(mask & ((1ull << lane) - 1ull))] = i;
    int all = 0;
    for (int k = 0; k < 16; ++k) all += wave_total[k];
    base += all;
    __syncthreads();
  }
}

__global__ __launch_bounds__(1024) void rank_select_kernel(const double* __restrict__ scores, int c, int keep,
                                                           int32_t* __restrict__ order,
                                                           int32_t* __restrict__ kept) {
  __shared__ double s[kMaxRankFilters];
  __shared__ int idx[kMaxRankFilters];
  __shared__ unsigned char alive[kMaxRankFilters];
  __shared__ int wave_total[16];
  rank_select(scores, c, keep, order, kept, s, idx, alive, wave_total);
}

__device__ __forceinline__ int clamp_index(int v, int n) { return v < 0 ? 0 : (v >= n ? n - 1 : v); }

// fp64 product -> fp32 (the folded weight as the fp32 path sees it) -> output type,
// both steps round-to-nearest-even.
template <typename T> __device__ __forceinline__ T round_from_f32(float f);
template <> __device__ __forceinline__ float round_from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ _Float16 round_from_f32<_Float16>(float f) { return (_Float16)f; }
template <> __device__ __forceinline__ __bf16 round_from_f32<__bf16>(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return __builtin_bit_cast(__bf16, (uint16_t)((u >> 16) | 0x40u));
  u += 0x7FFFu + ((u >> 16) & 1u);
  return __builtin_bit_cast(__bf16, (uint16_t)(u >> 16));
}
template <typename T> __device__ __forceinline__ T round_from_double(double v) {
  float f = (float)v;
  asm volatile("" : "+v"(f));  // keep the two roundings separate
  return round_from_f32<T>(f);
}

// ---- weight gather + fold ----------------------------------------------------------
// One layer's gather, as the kernels see it.
struct GatherJob {
  const float* w;                 // [c_out][c_in][khw]
  const int32_t* keep_out;        // [n_out] or null (all filters)
  const int32_t* keep_in;         // [n_in] or null (all channels)
  const float *gamma, *beta, *mean, *var, *conv_bias;   // null = absent
  void* w_out;                    // [n_out][n_in][khw]
  float* bias_out;                // [n_out] or null
  int c_out, c_in, khw, n_out, n_in;
  unsigned magic_khw;             // ceil(2^32 / khw): e / khw == umulhi(e, magic) for e * khw < 2^32
  int staged;                     // 1: a source row fits the LDS stage (c_in * khw <= kRowLds)
  int slices;                     // work-groups per output row (1 when staged)
  int block0;                     // plan: index of the layer's first work-group
  double eps;
};

// The fold factor and bias of output row i (filter o of the source), in fp64, contraction off.
__device__ __forceinline__ void fold_terms(const GatherJob& g, int o, double* s_out, double* b_out) {
#pragma clang fp contract(off)
  const double cb = g.conv_bias ? (double)g.conv_bias[o] : 0.0;
  double s = 1.0, b = cb;
  if (g.gamma) {
    s = (double)g.gamma[o] / sqrt((double)g.var[o] + g.eps);
    b = (double)g.beta[o] + (cb - (double)g.mean[o]) * s;
  }
  *s_out = s; *b_out = b;
}

// Output row i of a layer (slice `slice` of `g.slices`).  Staged form: the whole source row
// travels to LDS in consecutive 16-byte pieces, the kept columns are picked from there and
// stored in consecutive addresses; the division of an output index into (channel, tap) is a
// multiply-high.  Unstaged (rows longer than the stage): the same arithmetic straight from
// global memory.
template <typename T>
__device__ __forceinline__ void gather_row(const GatherJob& g, int i, int slice, float* row, double* terms) {
#pragma clang fp contract(off)
  const int o = g.keep_out ? clamp_index(g.keep_out[i], g.c_out) : i;
  if (threadIdx.x == 0) fold_terms(g, o, &terms[0], &terms[1]);
  const long src_row = (long)g.c_in * g.khw;
  const float* src = g.w + (long)o * src_row;
  if (g.staged) {
    if (((src_row & 3) == 0) && ((reinterpret_cast<uintptr_t>(src) & 15) == 0)) {
      const float4* s4 = reinterpret_cast<const float4*>(src);
      float4* r4 = reinterpret_cast<float4*>(row);
      for (int e = threadIdx.x; e < (int)(src_row >> 2); e += 256) r4[e] = s4[e];
    } else {
      for (int e = threadIdx.x; e < (int)src_row; e += 256) row[e] = src[e];
    }
  }
  __syncthreads();
  const double s = terms[0];
  if (g.bias_out && slice == 0 && threadIdx.x == 0) g.bias_out[i] = (float)terms[1];
  const unsigned out_row = (unsigned)g.n_in * (unsigned)g.khw;
  T* dst = reinterpret_cast<T*>(g.w_out) + (long)i * out_row;
  for (unsigned e = (unsigned)slice * 256u + threadIdx.x; e < out_row; e += (unsigned)g.slices * 256u) {
    unsigned se = e;
    if (g.keep_in) {
      const unsigned c = g.khw == 1 ? e : __umulhi(e, g.magic_khw);
      const unsigned t = e - c * (unsigned)g.khw;
      se = (unsigned)clamp_index(g.keep_in[c], g.c_in) * (unsigned)g.khw + t;
    }
    const float v = g.staged ? row[se] : src[se];
    dst[e] = round_from_double<T>((double)v * s);
  }
}

// dynamic LDS: the staged source row (as long as the launch's longest; more work-groups fit a compute unit
// when rows are short)
template <typename T>
__global__ __launch_bounds__(256) void gather_fold_kernel(GatherJob g) {
  extern __shared__ __align__(16) float row[];
  __shared__ double terms[2];
  gather_row<T>(g, blockIdx.x, blockIdx.y, row, terms);
}

// ---- plan kernels --------------------------------------------------------------------
struct ScoreMember { const float* w; long per_filter; };
struct RankJob {
  int c, keep;
  int first_member, n_members;   // into the plan's member list, in the order the sums are added
  int score0;                    // offset of the group's scores in the plan's score buffer
  int wave0;                     // index of the group's first wavefront in the scoring grid
  int32_t* kept;
};

// One wavefront per (ranked group, filter): the filter's L1 sum in every member, added in member order.
__global__ __launch_bounds__(256) void plan_score_kernel(const RankJob* __restrict__ jobs, int n_jobs,
                                                         const ScoreMember* __restrict__ members,
                                                         double* __restrict__ scores, int n_waves) {
  const int wv = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wv >= n_waves) return;
  int lo = 0, hi = n_jobs - 1;           // last job whose wave0 <= wv
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (jobs[mid].wave0 <= wv) lo = mid; else hi = mid - 1;
  }
  const RankJob jb = jobs[lo];
  const int j = wv - jb.wave0;
  if (j >= jb.c) return;
  double total = 0.0;
  for (int m = 0; m < jb.n_members; ++m) {
    const ScoreMember mem = members[jb.first_member + m];
    const double s = wave_sum(l1_lane_sum(mem.w + (long)j * mem.per_filter, mem.per_filter, threadIdx.x & 63, 64));
    total = m == 0 ? s : total + s;
  }
  if ((threadIdx.x & 63) == 0) scores[jb.score0 + j] = total;
}

__global__ __launch_bounds__(1024) void plan_rank_kernel(const RankJob* __restrict__ jobs,
                                                         const double* __restrict__ scores) {
  __shared__ double s[kMaxRankFilters];
  __shared__ int idx[kMaxRankFilters];
  __shared__ unsigned char alive[kMaxRankFilters];
  __shared__ int wave_total[16];
  const RankJob jb = jobs[blockIdx.x];
  rank_select(scores + jb.score0, jb.c, jb.keep, nullptr, jb.kept, s, idx, alive, wave_total);
}

template <typename T>
__global__ __launch_bounds__(256) void plan_gather_kernel(const GatherJob* __restrict__ jobs, int n_jobs) {
  extern __shared__ __align__(16) float row[];
  __shared__ double terms[2];
  const int b = blockIdx.x;
  int lo = 0, hi = n_jobs - 1;           // last job whose block0 <= b
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (jobs[mid].block0 <= b) lo = mid; else hi = mid - 1;
  }
  const GatherJob g = jobs[lo];
  const int r = b - g.block0;
  const int i = r / g.slices;
  gather_row<T>(g, i, r - i * g.slices, row, terms);
}

template <typename T>
__global__ __launch_bounds__(256) void gather_channels_kernel(const T* __restrict__ x, int c, long hw,
                                                              const int32_t* __restrict__ idx,
                                                              int n_idx, T* __restrict__ y) {
  // grid.x = n * n_idx (one output plane each), grid.y slices the plane
  const int plane = blockIdx.x;
  const int b = plane / n_idx, i = plane - b * n_idx;
  const int ci = clamp_index(idx[i], c);
  const T* src = x + ((long)b * c + ci) * hw;
  T* dst = y + (long)plane * hw;
  for (long e = (long)blockIdx.y * 256 + threadIdx.x; e < hw; e += (long)gridDim.y * 256) dst[e] = src[e];
}

// ---- host helpers ----------------------------------------------------------------------
int launch_scores(const float* w, long per_filter, int c_out, double* scores, int accumulate, hipStream_t s) {
  if (per_filter > kWaveFilterMax)
    hipLaunchKernelGGL(l1_score_group_kernel, dim3(c_out), dim3(256), 0, s, w, per_filter, scores, accumulate);
  else
    hipLaunchKernelGGL(l1_score_wave_kernel, dim3((c_out + 3) / 4), dim3(256), 0, s, w, per_filter, c_out, scores,
                       accumulate);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

// Fills the shape-derived fields of a gather job; CPRUNE_ERR_UNSUPPORTED for rows the 32-bit
// index arithmetic cannot address.
int finish_gather_job(GatherJob* g) {
  const long src_row = (long)g->c_in * g->khw, out_row = (long)g->n_in * g->khw;
  if (src_row * g->khw >= (1L << 32) || out_row >= (1L << 31)) return CPRUNE_ERR_UNSUPPORTED;
  g->magic_khw = g->khw > 1 ? (unsigned)((0x100000000ull + (unsigned)g->khw - 1) / (unsigned)g->khw) : 0u;
  g->staged = src_row <= kRowLds ? 1 : 0;
  int slices = 1;
  if (!g->staged || g->n_out < 256) {       // few or long rows: several work-groups share a row
    slices = (int)((out_row + 2047) / 2048);
    if (slices < 1) slices = 1;
    if (slices > 64) slices = 64;
    if (g->staged && slices > 4) slices = 4;   // every slice stages the whole source row
  }
  g->slices = slices;
  return CPRUNE_OK;
}

}  // namespace
}  // namespace cprune

using namespace cprune;

// Scores of the allocation-free ranking call: one array per device, held for the life of the process.
// In host code the name below is only a handle for hipGetSymbolAddress; kernels get the device address.
static __device__ __align__(256) double scratch[4096];

namespace {
constexpr int kStaticRankFilters = 4096;   // entries of `scratch`
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};

// The device address of `scratch` on the current device (looked up once per device).
int scratch_for_current_device(double** out) {
  int dev = -1;
  CPRUNE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CPRUNE_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    CPRUNE_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return CPRUNE_ERR_DEVICE;
    g_scratch_ptr[dev] = static_cast<double*>(p);
  }
  *out = g_scratch_ptr[dev];
  return CPRUNE_OK;
}
}  // namespace

extern "C" size_t cprune_rank_filters_workspace_bytes(int c_out) {
  return c_out > 0 ? (size_t)c_out * sizeof(double) : 0;
}

extern "C" int cprune_rank_filters(const float* w, int c_out, int c_in_per_group, int kh, int kw,
                                   int keep, double* scores_out, int32_t* order_out,
                                   int32_t* kept_out, void* ws, size_t ws_bytes, void* stream) {
  if (!w || !kept_out || c_out < 1 || c_in_per_group < 1 || kh < 1 || kw < 1) return CPRUNE_ERR_INVALID_ARG;
  if (keep < 1 || keep > c_out) return CPRUNE_ERR_INVALID_ARG;
  if (c_out > kMaxRankFilters) return CPRUNE_ERR_UNSUPPORTED;
  double* scores = scores_out;
  if (!scores) {
    if (!ws) return CPRUNE_ERR_INVALID_ARG;
    if (ws_bytes < cprune_rank_filters_workspace_bytes(c_out)) return CPRUNE_ERR_WORKSPACE;
    scores = (double*)ws;
  }
  hipStream_t s = (hipStream_t)stream;
  int rc = launch_scores(w, (long)c_in_per_group * kh * kw, c_out, scores, 0, s);
  if (rc != CPRUNE_OK) return rc;
  hipLaunchKernelGGL(rank_select_kernel, dim3(1), dim3(1024), 0, s, scores, c_out, keep, order_out,
                     kept_out);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

extern "C" int cprune_rank_filters_static(const float* w, int c_out, int c_in_per_group, int kh, int kw,
                                          int keep, int32_t* order_out, int32_t* kept_out, void* stream) {
  if (!w || !kept_out || c_out < 1 || c_in_per_group < 1 || kh < 1 || kw < 1) return CPRUNE_ERR_INVALID_ARG;
  if (keep < 1 || keep > c_out) return CPRUNE_ERR_INVALID_ARG;
  if (c_out > kStaticRankFilters) return CPRUNE_ERR_UNSUPPORTED;   // more filters than the static array holds
  double* scores = nullptr;
  int rc = scratch_for_current_device(&scores);
  if (rc != CPRUNE_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  // every score the ranking reads is written by the scoring launch in front of it: nothing to clear
  rc = launch_scores(w, (long)c_in_per_group * kh * kw, c_out, scores, 0, s);
  if (rc != CPRUNE_OK) return rc;
  hipLaunchKernelGGL(rank_select_kernel, dim3(1), dim3(1024), 0, s, scores, c_out, keep, order_out, kept_out);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

extern "C" int cprune_rank_filters_static_max(void) { return kStaticRankFilters; }

extern "C" int cprune_rank_filter_group(const float* const* w, const int64_t* per_filter, int n_members,
                                        int c_out, int keep, double* scores_out, int32_t* order_out,
                                        int32_t* kept_out, void* ws, size_t ws_bytes, void* stream) {
  if (!w || !per_filter || n_members < 1 || !kept_out || c_out < 1) return CPRUNE_ERR_INVALID_ARG;
  for (int m = 0; m < n_members; ++m)
    if (!w[m] || per_filter[m] < 1) return CPRUNE_ERR_INVALID_ARG;
  if (keep < 1 || keep > c_out) return CPRUNE_ERR_INVALID_ARG;
  if (c_out > kMaxRankFilters) return CPRUNE_ERR_UNSUPPORTED;
  double* scores = scores_out;
  if (!scores) {
    if (!ws) return CPRUNE_ERR_INVALID_ARG;
    if (ws_bytes < cprune_rank_filters_workspace_bytes(c_out)) return CPRUNE_ERR_WORKSPACE;
    scores = (double*)ws;
  }
  hipStream_t s = (hipStream_t)stream;
  for (int m = 0; m < n_members; ++m) {   // same stream: member m + 1 adds to what member m left
    int rc = launch_scores(w[m], (long)per_filter[m], c_out, scores, m > 0 ? 1 : 0, s);
    if (rc != CPRUNE_OK) return rc;
  }
  hipLaunchKernelGGL(rank_select_kernel, dim3(1), dim3(1024), 0, s, scores, c_out, keep, order_out, kept_out);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

extern "C" int cprune_gather_pruned_weights(const float* w, int c_out, int c_in, int kh, int kw,
                                            const int32_t* keep_out, int n_keep_out,
                                            const int32_t* keep_in, int n_keep_in,
                                            const float* gamma, const float* beta,
                                            const float* mean, const float* var, float eps,
                                            const float* conv_bias, cprune_dtype out_dtype,
                                            void* w_out, float* bias_out, void* stream) {
  if (!w || !w_out || c_out < 1 || c_in < 1 || kh < 1 || kw < 1) return CPRUNE_ERR_INVALID_ARG;
  if (!dtype_ok(out_dtype)) return CPRUNE_ERR_INVALID_ARG;
  const int n_out = keep_out ? n_keep_out : c_out;
  const int n_in = keep_in ? n_keep_in : c_in;
  if (n_out < 1 || n_out > c_out || n_in < 1 || n_in > c_in) return CPRUNE_ERR_INVALID_ARG;
  const bool any_bn = gamma || beta || mean || var;
  const bool all_bn = gamma && beta && mean && var;
  if (any_bn && !all_bn) return CPRUNE_ERR_INVALID_ARG;
  if ((any_bn || conv_bias) && !bias_out) return CPRUNE_ERR_INVALID_ARG;
  if (any_bn && !(eps >= 0.0f)) return CPRUNE_ERR_INVALID_ARG;
  if ((long)kh * kw >= (1L << 15)) return CPRUNE_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  GatherJob g;
  g.w = w; g.keep_out = keep_out; g.keep_in = keep_in;
  g.gamma = gamma; g.beta = beta; g.mean = mean; g.var = var; g.conv_bias = conv_bias;
  g.w_out = w_out; g.bias_out = bias_out;
  g.c_out = c_out; g.c_in = c_in; g.khw = kh * kw; g.n_out = n_out; g.n_in = n_in;
  g.block0 = 0; g.eps = (double)eps;
  int rc = finish_gather_job(&g);
  if (rc != CPRUNE_OK) return rc;
  dim3 grid((unsigned)n_out, (unsigned)g.slices);
  const size_t lds = g.staged ? (size_t)c_in * g.khw * sizeof(float) : 0;
  if (out_dtype == CPRUNE_F32) hipLaunchKernelGGL(gather_fold_kernel<float>, grid, dim3(256), lds, s, g);
  else if (out_dtype == CPRUNE_F16) hipLaunchKernelGGL(gather_fold_kernel<_Float16>, grid, dim3(256), lds, s, g);
  else hipLaunchKernelGGL(gather_fold_kernel<__bf16>, grid, dim3(256), lds, s, g);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

// ---- whole-network plan ---------------------------------------------------------------
struct cprune_prune_plan {
  std::vector<RankJob> rank_jobs;
  std::vector<GatherJob> gather_jobs;
  RankJob* d_rank_jobs = nullptr;
  ScoreMember* d_members = nullptr;
  GatherJob* d_gather_jobs = nullptr;
  double* d_scores = nullptr;
  int n_waves = 0, n_blocks = 0, dtype = CPRUNE_F32;
  size_t gather_lds = 0;   // bytes of the longest source row any layer stages
  long weights_read = 0, weights_written = 0;   // elements
};

static void plan_free(cprune_prune_plan* p) {
  if (p->d_rank_jobs) hipFree(p->d_rank_jobs);
  if (p->d_members) hipFree(p->d_members);
  if (p->d_gather_jobs) hipFree(p->d_gather_jobs);
  if (p->d_scores) hipFree(p->d_scores);
  delete p;
}

extern "C" int cprune_prune_plan_create(const cprune_prune_layer* layers, int n_layers, float eps,
                                        cprune_dtype out_dtype, cprune_prune_plan** out) {
  if (!layers || !out || n_layers < 1 || !dtype_ok(out_dtype) || !(eps >= 0.0f)) return CPRUNE_ERR_INVALID_ARG;
  // validation: shapes, references to earlier ranked layers, pointers
  for (int i = 0; i < n_layers; ++i) {
    const cprune_prune_layer& L = layers[i];
    if (!L.w) {   // a layer without weights (a pool): placeholder, nothing may refer to it
      if (L.keep != 0 || L.rows_from >= 0 || L.cols_from >= 0 || L.n_score_with != 0) return CPRUNE_ERR_INVALID_ARG;
      continue;
    }
    if (L.c_out < 1 || L.c_in < 1 || L.kh < 1 || L.kw < 1 || !L.w_out) return CPRUNE_ERR_INVALID_ARG;
    if ((long)L.kh * L.kw >= (1L << 15)) return CPRUNE_ERR_UNSUPPORTED;
    if (L.keep < 0 || L.keep > L.c_out) return CPRUNE_ERR_INVALID_ARG;
    if (L.keep > 0) {
      if (!L.kept_out || L.rows_from != i || L.n_score_with < 0) return CPRUNE_ERR_INVALID_ARG;
      if (L.c_out > kMaxRankFilters) return CPRUNE_ERR_UNSUPPORTED;
      if (L.n_score_with > 0 && !L.score_with) return CPRUNE_ERR_INVALID_ARG;
      for (int m = 0; m < L.n_score_with; ++m) {
        const int j = L.score_with[m];
        if (j < 0 || j >= n_layers || j == i || !layers[j].w || layers[j].c_out != L.c_out) return CPRUNE_ERR_INVALID_ARG;
      }
    } else if (L.n_score_with != 0) {
      return CPRUNE_ERR_INVALID_ARG;
    }
    const int refs[2] = {L.rows_from, L.cols_from};
    for (int r = 0; r < 2; ++r) {
      const int j = refs[r];
      if (j < -1 || j >= n_layers) return CPRUNE_ERR_INVALID_ARG;
      if (j >= 0 && (layers[j].keep < 1 || !layers[j].w)) return CPRUNE_ERR_INVALID_ARG;   // must be a ranked layer
    }
    if (L.rows_from >= 0 && layers[L.rows_from].c_out != L.c_out) return CPRUNE_ERR_INVALID_ARG;
    if (L.cols_from >= 0 && layers[L.cols_from].c_out != L.c_in) return CPRUNE_ERR_INVALID_ARG;
    const bool any_bn = L.gamma || L.beta || L.mean || L.var;
    const bool all_bn = L.gamma && L.beta && L.mean && L.var;
    if (any_bn && !all_bn) return CPRUNE_ERR_INVALID_ARG;
    if ((any_bn || L.conv_bias) && !L.bias_out) return CPRUNE_ERR_INVALID_ARG;
  }
  cprune_prune_plan* p = new cprune_prune_plan();
  p->dtype = out_dtype;
  std::vector<ScoreMember> members;
  int n_scores = 0;
  for (int i = 0; i < n_layers; ++i) {
    const cprune_prune_layer& L = layers[i];
    if (!L.w || L.keep < 1) continue;
    RankJob jb;
    jb.c = L.c_out; jb.keep = L.keep; jb.first_member = (int)members.size(); jb.n_members = 1 + L.n_score_with;
    jb.score0 = n_scores; jb.wave0 = p->n_waves; jb.kept = L.kept_out;
    members.push_back(ScoreMember{L.w, (long)L.c_in * L.kh * L.kw});
    for (int m = 0; m < L.n_score_with; ++m) {
      const cprune_prune_layer& M = layers[L.score_with[m]];
      members.push_back(ScoreMember{M.w, (long)M.c_in * M.kh * M.kw});
    }
    for (int m = 0; m < jb.n_members; ++m) p->weights_read += (long)L.c_out * members[jb.first_member + m].per_filter;
    n_scores += L.c_out;
    p->n_waves += (L.c_out + 3) / 4 * 4;     // a group's filters start on a work-group boundary
    p->rank_jobs.push_back(jb);
  }
  int rc = CPRUNE_OK;
  for (int i = 0; i < n_layers && rc == CPRUNE_OK; ++i) {
    const cprune_prune_layer& L = layers[i];
    if (!L.w) continue;
    GatherJob g;
    g.w = L.w;
    g.keep_out = L.rows_from >= 0 ? layers[L.rows_from].kept_out : nullptr;
    g.keep_in = L.cols_from >= 0 ? layers[L.cols_from].kept_out : nullptr;
    g.gamma = L.gamma; g.beta = L.beta; g.mean = L.mean; g.var = L.var; g.conv_bias = L.conv_bias;
    g.w_out = L.w_out; g.bias_out = L.bias_out;
    g.c_out = L.c_out; g.c_in = L.c_in; g.khw = L.kh * L.kw;
    g.n_out = L.rows_from >= 0 ? layers[L.rows_from].keep : L.c_out;
    g.n_in = L.cols_from >= 0 ? layers[L.cols_from].keep : L.c_in;
    g.eps = (double)eps;
    rc = finish_gather_job(&g);
    if (g.staged) p->gather_lds = std::max(p->gather_lds, (size_t)g.c_in * g.khw * sizeof(float));
    g.block0 = p->n_blocks;
    p->n_blocks += g.n_out * g.slices;
    p->weights_read += (long)g.n_out * g.c_in * g.khw;
    p->weights_written += (long)g.n_out * g.n_in * g.khw;
    p->gather_jobs.push_back(g);
  }
  auto upload = [&](const void* src, size_t bytes, void** dst) -> int {
    hipError_t e = hipMalloc(dst, bytes ? bytes : 16);
    if (e == hipSuccess && bytes) e = hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
    return CPRUNE_OK;
  };
  if (rc == CPRUNE_OK) rc = upload(p->rank_jobs.data(), p->rank_jobs.size() * sizeof(RankJob), (void**)&p->d_rank_jobs);
  if (rc == CPRUNE_OK) rc = upload(members.data(), members.size() * sizeof(ScoreMember), (void**)&p->d_members);
  if (rc == CPRUNE_OK) rc = upload(p->gather_jobs.data(), p->gather_jobs.size() * sizeof(GatherJob), (void**)&p->d_gather_jobs);
  if (rc == CPRUNE_OK) {
    hipError_t e = hipMalloc((void**)&p->d_scores, (size_t)(n_scores > 0 ? n_scores : 1) * sizeof(double));
    if (e != hipSuccess) { set_last_hip_error(e); rc = CPRUNE_ERR_DEVICE; }
  }
  if (rc != CPRUNE_OK) { plan_free(p); return rc; }
  *out = p;
  return CPRUNE_OK;
}

extern "C" int cprune_prune_plan_run(cprune_prune_plan* p, void* stream) {
  if (!p) return CPRUNE_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int n_rank = (int)p->rank_jobs.size(), n_gather = (int)p->gather_jobs.size();
  if (n_rank > 0) {
    hipLaunchKernelGGL(plan_score_kernel, dim3(p->n_waves / 4), dim3(256), 0, s, p->d_rank_jobs, n_rank, p->d_members,
                       p->d_scores, p->n_waves);
    CPRUNE_LAUNCH_CHECK();
    hipLaunchKernelGGL(plan_rank_kernel, dim3(n_rank), dim3(1024), 0, s, p->d_rank_jobs, p->d_scores);
    CPRUNE_LAUNCH_CHECK();
  }
  if (n_gather > 0) {
    dim3 grid((unsigned)p->n_blocks);
    const size_t lds = p->gather_lds;
    if (p->dtype == CPRUNE_F32) hipLaunchKernelGGL(plan_gather_kernel<float>, grid, dim3(256), lds, s, p->d_gather_jobs, n_gather);
    else if (p->dtype == CPRUNE_F16) hipLaunchKernelGGL(plan_gather_kernel<_Float16>, grid, dim3(256), lds, s, p->d_gather_jobs, n_gather);
    else hipLaunchKernelGGL(plan_gather_kernel<__bf16>, grid, dim3(256), lds, s, p->d_gather_jobs, n_gather);
    CPRUNE_LAUNCH_CHECK();
  }
  return CPRUNE_OK;
}

extern "C" int cprune_prune_plan_traffic(const cprune_prune_plan* p, int64_t* weights_read_out,
                                         int64_t* weights_written_out) {
  if (!p || !weights_read_out || !weights_written_out) return CPRUNE_ERR_INVALID_ARG;
  *weights_read_out = p->weights_read;
  *weights_written_out = p->weights_written;
  return CPRUNE_OK;
}

extern "C" int cprune_prune_plan_destroy(cprune_prune_plan* p) {
  if (!p) return CPRUNE_ERR_INVALID_ARG;
  hipError_t e = hipDeviceSynchronize();
  plan_free(p);
  if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
  return CPRUNE_OK;
}

extern "C" int cprune_gather_channels(const void* x, int n, int c, int h, int w, cprune_dtype dtype,
                                      const int32_t* idx, int n_idx, void* y, void* stream) {
  if (!x || !y || !idx || n < 1 || c < 1 || h < 1 || w < 1) return CPRUNE_ERR_INVALID_ARG;
  if (n_idx < 1 || n_idx > c || !dtype_ok(dtype)) return CPRUNE_ERR_INVALID_ARG;
  if ((long)n * c * h * w >= (1L << 31)) return CPRUNE_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  const long hw = (long)h * w;
  int slices = (int)((hw + 1023) / 1024);
  if (slices > 256) slices = 256;
  dim3 grid((unsigned)(n * n_idx), (unsigned)slices);
  if (dtype == CPRUNE_F32)
    hipLaunchKernelGGL(gather_channels_kernel<float>, grid, dim3(256), 0, s, (const float*)x, c, hw,
                       idx, n_idx, (float*)y);
  else
    hipLaunchKernelGGL(gather_channels_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t*)x,
                       c, hw, idx, n_idx, (uint16_t*)y);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}
