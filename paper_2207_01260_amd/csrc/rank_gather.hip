// Filter ranking and channel gather (paper Section 3.5, last paragraph, and
// Section 2.1): L1 score per filter, rank by (score descending, index
// ascending), ascending kept list, weight gather with batch-norm folding,
// activation channel gather.  All bandwidth- or latency-bound; none of it is a
// contraction, so none of it uses the matrix cores.
#include "common.hpp"

namespace cprune {
namespace {

constexpr int kMaxRankFilters = 4096;

// One work-group per filter.  Each thread adds |w| over a strided slice in
// double, then a fixed-shape tree (wavefront shuffles, then 4 partials in LDS)
// combines them: the order of additions depends only on the filter length, so
// the score is reproducible bit for bit.
// accumulate != 0: the sum is added to the score already there (groups of layers).
__global__ __launch_bounds__(256) void l1_score_kernel(const float* __restrict__ w, long per_filter,
                                                       double* __restrict__ scores, int accumulate) {
  const float* f = w + (long)blockIdx.x * per_filter;
  double s = 0.0;
  for (long i = threadIdx.x; i < per_filter; i += 256) s += (double)fabsf(f[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
  __shared__ double part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    const double sum = (part[0] + part[1]) + (part[2] + part[3]);
    scores[blockIdx.x] = accumulate ? scores[blockIdx.x] + sum : sum;
  }
}

// Enumeration sort in one work-group: rank(i) = #{ j : s_j > s_i or (s_j == s_i and j < i) }.
// order[rank(i)] = i; filter i survives iff rank(i) < keep; its slot in the
// ascending kept list is the number of surviving filters with a lower index.
__global__ __launch_bounds__(1024) void rank_select_kernel(const double* __restrict__ scores, int c,
                                                           int keep, int32_t* __restrict__ order,
                                                           int32_t* __restrict__ kept) {
  __shared__ double s[kMaxRankFilters];
  __shared__ unsigned char alive[kMaxRankFilters];
  for (int i = threadIdx.x; i < c; i += 1024) s[i] = scores[i];
  __syncthreads();
  for (int i = threadIdx.x; i < c; i += 1024) {
    double si = s[i];
    int rank = 0;
    for (int j = 0; j < c; ++j) {
      double sj = s[j];
      rank += (sj > si || (sj == si && j < i)) ? 1 : 0;
    }
    if (order) order[rank] = i;
    alive[i] = rank < keep;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < c; i += 1024) {
    if (!alive[i]) continue;
    int pos = 0;
    for (int j = 0; j < i; ++j) pos += alive[j];
    kept[pos] = i;
  }
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

// One work-group per kept filter (grid.x) and slice of its row (grid.y).
template <typename T>
__global__ __launch_bounds__(256) void gather_fold_kernel(
    const float* __restrict__ w, int c_out, int c_in, int khw, const int32_t* __restrict__ keep_out,
    const int32_t* __restrict__ keep_in, int n_in, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ mean, const float* __restrict__ var,
    double eps, const float* __restrict__ conv_bias, T* __restrict__ w_out,
    float* __restrict__ bias_out) {
#pragma clang fp contract(off)
  const int i = blockIdx.x;
  const int o = keep_out ? clamp_index(keep_out[i], c_out) : i;
  const double cb = conv_bias ? (double)conv_bias[o] : 0.0;
  double s = 1.0, b = cb;
  if (gamma) {
    s = (double)gamma[o] / sqrt((double)var[o] + eps);
    b = (double)beta[o] + (cb - (double)mean[o]) * s;
  }
  if (bias_out && blockIdx.y == 0 && threadIdx.x == 0) bias_out[i] = (float)b;
  const long row = (long)n_in * khw;
  const float* src = w + (long)o * c_in * khw;
  T* dst = w_out + (long)i * row;
  for (long e = (long)blockIdx.y * 256 + threadIdx.x; e < row; e += (long)gridDim.y * 256) {
    long se = e;
    if (keep_in) {
      int c = (int)(e / khw);
      int t = (int)(e - (long)c * khw);
      se = (long)clamp_index(keep_in[c], c_in) * khw + t;
    }
    dst[e] = round_from_double<T>((double)src[se] * s);
  }
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

}  // namespace
}  // namespace cprune

using namespace cprune;

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
  long per_filter = (long)c_in_per_group * kh * kw;
  hipLaunchKernelGGL(l1_score_kernel, dim3(c_out), dim3(256), 0, s, w, per_filter, scores, 0);
  CPRUNE_LAUNCH_CHECK();
  hipLaunchKernelGGL(rank_select_kernel, dim3(1), dim3(1024), 0, s, scores, c_out, keep, order_out,
                     kept_out);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

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
    hipLaunchKernelGGL(l1_score_kernel, dim3(c_out), dim3(256), 0, s, w[m], (long)per_filter[m], scores, m > 0 ? 1 : 0);
    CPRUNE_LAUNCH_CHECK();
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
  hipStream_t s = (hipStream_t)stream;
  const int khw = kh * kw;
  const long row = (long)n_in * khw;
  int slices = (int)((row + 2047) / 2048);
  if (slices < 1) slices = 1;
  if (slices > 64) slices = 64;
  dim3 grid((unsigned)n_out, (unsigned)slices);
#define GO(T)                                                                                   \
  hipLaunchKernelGGL(gather_fold_kernel<T>, grid, dim3(256), 0, s, w, c_out, c_in, khw, keep_out, \
                     keep_in, n_in, gamma, beta, mean, var, (double)eps, conv_bias, (T*)w_out,  \
                     bias_out)
  if (out_dtype == CPRUNE_F32) GO(float);
  else if (out_dtype == CPRUNE_F16) GO(_Float16);
  else GO(__bf16);
#undef GO
  CPRUNE_LAUNCH_CHECK();
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
