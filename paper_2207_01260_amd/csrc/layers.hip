// Bandwidth-bound layers of the evaluated networks: depthwise convolution
// (MobileNetV2's 3x3 stage between the pruned 1x1 expansion and projection),
// max pooling and global average pooling.  No contraction across channels, so
// these are plain coalesced kernels: consecutive lanes take consecutive output
// columns of one (image, channel) plane.
#include "common.hpp"

namespace cprune {
namespace {

template <typename T> __device__ __forceinline__ float ld(const T* p) { return (float)*p; }
template <typename T> __device__ __forceinline__ void st(T* p, float v) { *p = (T)v; }

// an activation is a clamp with uniform bounds: a max and a min per element, no branches
__device__ __forceinline__ float act_f(float v, int act) {
  const float lo = act == CPRUNE_ACT_NONE ? -__builtin_inff() : 0.0f;
  const float hi = act == CPRUNE_ACT_RELU6 ? 6.0f : __builtin_inff();
  return fminf(fmaxf(v, lo), hi);
}

// grid.x = n*c planes, grid.y slices the output plane; weights of the plane's
// channel are read once into registers (k <= 7).
template <typename T, int K>
__global__ __launch_bounds__(256) void depthwise_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                        const float* __restrict__ bias,
                                                        const T* __restrict__ res, T* __restrict__ y,
                                                        int c, int h, int wd, int ho, int wo, int stride,
                                                        int pad, int act) {
  const int plane = blockIdx.x;
  const int ch = plane % c;
  float wk[K * K];
#pragma unroll
  for (int i = 0; i < K * K; ++i) wk[i] = ld(w + (long)ch * K * K + i);
  const float b = bias ? bias[ch] : 0.0f;
  const T* xp = x + (long)plane * h * wd;
  const long obase = (long)plane * ho * wo;
  const int total = ho * wo;
  for (int e = blockIdx.y * 256 + threadIdx.x; e < total; e += gridDim.y * 256) {
    int oy = e / wo, ox = e - oy * wo;
    int iy0 = oy * stride - pad, ix0 = ox * stride - pad;
    float acc = 0.0f;
#pragma unroll
    for (int u = 0; u < K; ++u) {
      int iy = iy0 + u;
      if ((unsigned)iy >= (unsigned)h) continue;
#pragma unroll
      for (int v = 0; v < K; ++v) {
        int ix = ix0 + v;
        if ((unsigned)ix < (unsigned)wd) acc += ld(xp + (long)iy * wd + ix) * wk[u * K + v];
      }
    }
    acc += b;
    if (res) acc += ld(res + obase + e);
    st(y + obase + e, act_f(acc, act));
  }
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool_kernel(const T* __restrict__ x, T* __restrict__ y, int h,
                                                      int wd, int ho, int wo, int k, int stride,
                                                      int pad) {
  const int plane = blockIdx.x;
  const T* xp = x + (long)plane * h * wd;
  const int total = ho * wo;
  for (int e = blockIdx.y * 256 + threadIdx.x; e < total; e += gridDim.y * 256) {
    int oy = e / wo, ox = e - oy * wo;
    int iy0 = oy * stride - pad, ix0 = ox * stride - pad;
    float m = 0.0f;
    bool have = false;
    for (int u = 0; u < k; ++u) {
      int iy = iy0 + u;
      if ((unsigned)iy >= (unsigned)h) continue;
      for (int v = 0; v < k; ++v) {
        int ix = ix0 + v;
        if ((unsigned)ix >= (unsigned)wd) continue;
        float val = ld(xp + (long)iy * wd + ix);
        if (!have || val > m) { m = val; have = true; }
      }
    }
    st(y + (long)plane * total + e, m);
  }
}

// One wavefront per (image, channel) plane: strided partial sums, then a
// shuffle tree; 4 planes per work-group.
template <typename T>
__global__ __launch_bounds__(256) void gavgpool_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                       int planes, int hw) {
  const int plane = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (plane >= planes) return;
  const int lane = threadIdx.x & 63;
  const T* xp = x + (long)plane * hw;
  float s = 0.0f;
  for (int i = lane; i < hw; i += 64) s += ld(xp + i);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
  if (lane == 0) st(y + plane, s / (float)hw);
}

// ---- channels-last twins used inside the network handle ------------------------
// One thread per output element, consecutive threads on consecutive channels of a
// pixel (the contiguous direction of [n][h][w][cp]); pad channels carry zeros.

template <typename T>
__global__ __launch_bounds__(256) void maxpool_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                           long total, int cp, int h, int wd, int ho, int wo,
                                                           int k, int stride, int pad) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cp);
  long pix = i / cp;
  const int ox = (int)(pix % wo); pix /= wo;
  const int oy = (int)(pix % ho);
  const long n = pix / ho;
  const int iy0 = oy * stride - pad, ix0 = ox * stride - pad;
  float m = 0.0f;
  bool have = false;
  for (int u = 0; u < k; ++u) {
    const int iy = iy0 + u;
    if ((unsigned)iy >= (unsigned)h) continue;
    for (int v = 0; v < k; ++v) {
      const int ix = ix0 + v;
      if ((unsigned)ix >= (unsigned)wd) continue;
      const float val = ld(x + ((n * h + iy) * wd + ix) * cp + c);
      if (!have || val > m) { m = val; have = true; }
    }
  }
  st(y + i, m);
}

template <typename T>
__global__ __launch_bounds__(256) void gavgpool_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                            int total, int cp, int hw) {
  const int i = blockIdx.x * 256 + threadIdx.x;  // (n, c)
  if (i >= total) return;
  const int c = i % cp;
  const long n = i / cp;
  const T* xp = x + n * hw * cp + c;
  float s = 0.0f;
  for (int p = 0; p < hw; ++p) s += ld(xp + (long)p * cp);
  st(y + i, s / (float)hw);
}

template <typename T, int K>
__global__ __launch_bounds__(256) void depthwise_nhwc_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                             const float* __restrict__ bias,
                                                             const T* __restrict__ res, T* __restrict__ y,
                                                             long total, int c_real, int cp, int h, int wd,
                                                             int ho, int wo, int stride, int pad, int act) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % cp);
  long pix = i / cp;
  const int ox = (int)(pix % wo); pix /= wo;
  const int oy = (int)(pix % ho);
  const long n = pix / ho;
  const int iy0 = oy * stride - pad, ix0 = ox * stride - pad;
  float acc = 0.0f;
#pragma unroll
  for (int u = 0; u < K; ++u) {
    const int iy = iy0 + u;
    if ((unsigned)iy >= (unsigned)h) continue;
#pragma unroll
    for (int v = 0; v < K; ++v) {
      const int ix = ix0 + v;
      if ((unsigned)ix < (unsigned)wd)
        acc += ld(x + ((n * h + iy) * wd + ix) * cp + c) * ld(w + (u * K + v) * cp + c);
    }
  }
  if (bias && c < c_real) acc += bias[c];
  if (res) acc += ld(res + i);
  st(y + i, act_f(acc, act));
}

// Channels-last depthwise, vectorised: a thread owns one 16-byte channel vector (4 floats /
// 8 halves) of TX neighbouring output pixels of a row.  Consecutive lanes take consecutive
// channel vectors, so every access is a coalesced 16-byte load or store; the K x K weights of
// the vector sit in registers; each input column loaded serves every output of the run whose
// window covers it ((TX - 1) * S + K loads per row for TX outputs instead of TX * K).
template <typename T> struct VecOf;
template <> struct VecOf<float> { static constexpr int V = 4; };
template <> struct VecOf<_Float16> { static constexpr int V = 8; };
template <> struct VecOf<__bf16> { static constexpr int V = 8; };

template <typename T, int V>
__device__ __forceinline__ void unpack16(const uint4& q, float (&f)[V]) {
  if constexpr (V == 4) {
    f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y); f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
  } else {
    const T* h = reinterpret_cast<const T*>(&q);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
  }
}

// Channels-last max-pool on 16-byte channel vectors (one output pixel and vector per thread).
template <typename T>
__global__ __launch_bounds__(256) void maxpool_nhwc_vec_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                               unsigned total, int cp, int h, int wd, int ho,
                                                               int wo, int k, int stride, int pad) {
  constexpr int V = VecOf<T>::V;
  const unsigned idx = blockIdx.x * 256u + threadIdx.x;
  if (idx >= total) return;
  const unsigned nvec = (unsigned)cp / V;
  const int c0 = (int)(idx % nvec) * V;
  unsigned r = idx / nvec;
  const int ox = (int)(r % (unsigned)wo); r /= (unsigned)wo;
  const int oy = (int)(r % (unsigned)ho);
  const int n = (int)(r / (unsigned)ho);
  float m[V];
  bool have = false;
  for (int u = 0; u < k; ++u) {
    const int iy = oy * stride - pad + u;
    if ((unsigned)iy >= (unsigned)h) continue;
    for (int v = 0; v < k; ++v) {
      const int ix = ox * stride - pad + v;
      if ((unsigned)ix >= (unsigned)wd) continue;
      float in[V];
      unpack16<T, V>(*reinterpret_cast<const uint4*>(x + ((size_t)(n * h + iy) * wd + ix) * cp + c0), in);
#pragma unroll
      for (int e = 0; e < V; ++e) m[e] = have ? fmaxf(m[e], in[e]) : in[e];
      have = true;
    }
  }
  uint4 q;
  if constexpr (V == 4) {
    q.x = __float_as_uint(m[0]); q.y = __float_as_uint(m[1]); q.z = __float_as_uint(m[2]); q.w = __float_as_uint(m[3]);
  } else {
    T* hq = reinterpret_cast<T*>(&q);
#pragma unroll
    for (int e = 0; e < 8; ++e) hq[e] = (T)m[e];
  }
  *reinterpret_cast<uint4*>(y + (size_t)idx * V) = q;
}

template <typename T, int K, int S, int TX>
__global__ __launch_bounds__(256) void depthwise_nhwc_vec_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                                 const float* __restrict__ bias,
                                                                 const T* __restrict__ res, T* __restrict__ y,
                                                                 unsigned total, int c_real, int cp, int h, int wd,
                                                                 int ho, int wo, int xblocks, int pad, int act) {
  constexpr int V = VecOf<T>::V;
  constexpr int NIN = (TX - 1) * S + K;
  const unsigned idx = blockIdx.x * 256u + threadIdx.x;
  if (idx >= total) return;
  const unsigned nvec = (unsigned)cp / V;
  const unsigned cv = idx % nvec;
  unsigned r = idx / nvec;
  const int xb = (int)(r % (unsigned)xblocks); r /= (unsigned)xblocks;
  const int oy = (int)(r % (unsigned)ho);
  const int n = (int)(r / (unsigned)ho);
  const int c0 = (int)cv * V;

  float wk[K * K][V];
#pragma unroll
  for (int i = 0; i < K * K; ++i) unpack16<T, V>(*reinterpret_cast<const uint4*>(w + (size_t)i * cp + c0), wk[i]);
  float acc[TX][V];
#pragma unroll
  for (int t = 0; t < TX; ++t)
#pragma unroll
    for (int e = 0; e < V; ++e) acc[t][e] = 0.0f;

  const int ox0 = xb * TX;
  const int ix_base = ox0 * S - pad;
#pragma unroll
  for (int u = 0; u < K; ++u) {
    const int iy = oy * S - pad + u;
    if ((unsigned)iy >= (unsigned)h) continue;
    const T* row = x + ((size_t)(n * h + iy) * wd) * cp + c0;
#pragma unroll
    for (int j = 0; j < NIN; ++j) {
      const int ix = ix_base + j;
      float in[V];
      if ((unsigned)ix < (unsigned)wd) {
        unpack16<T, V>(*reinterpret_cast<const uint4*>(row + (size_t)ix * cp), in);
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) in[e] = 0.0f;
      }
#pragma unroll
      for (int t = 0; t < TX; ++t) {
        const int v = j - t * S;
        if (v >= 0 && v < K) {
#pragma unroll
          for (int e = 0; e < V; ++e) acc[t][e] += in[e] * wk[u * K + v][e];
        }
      }
    }
  }
  float bv[V];
#pragma unroll
  for (int e = 0; e < V; ++e) bv[e] = (bias && c0 + e < c_real) ? bias[c0 + e] : 0.0f;
#pragma unroll
  for (int t = 0; t < TX; ++t) {
    const int ox = ox0 + t;
    if (ox >= wo) break;
    const size_t off = ((size_t)(n * ho + oy) * wo + ox) * cp + c0;
    float o[V];
#pragma unroll
    for (int e = 0; e < V; ++e) o[e] = acc[t][e] + bv[e];
    if (res) {
      float rv[V];
      unpack16<T, V>(*reinterpret_cast<const uint4*>(res + off), rv);
#pragma unroll
      for (int e = 0; e < V; ++e) o[e] += rv[e];
    }
    uint4 q;
    if constexpr (V == 4) {
      q.x = __float_as_uint(act_f(o[0], act)); q.y = __float_as_uint(act_f(o[1], act));
      q.z = __float_as_uint(act_f(o[2], act)); q.w = __float_as_uint(act_f(o[3], act));
    } else {
      T* hq = reinterpret_cast<T*>(&q);
#pragma unroll
      for (int e = 0; e < 8; ++e) hq[e] = (T)act_f(o[e], act);
    }
    *reinterpret_cast<uint4*>(y + off) = q;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void nchw_to_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                           long total, int c, int hw, int cp) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int ch = (int)(i % cp);
  const long pix = i / cp;
  const long n = pix / hw;
  const int p = (int)(pix - n * hw);
  T v = (T)0.0f;
  if (ch < c) v = x[(n * c + ch) * hw + p];
  y[i] = v;
}

template <typename T>
__global__ __launch_bounds__(256) void nhwc_to_nchw_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                           long total, int c, int hw, int cp) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;  // index into dense [n][c][hw]
  if (i >= total) return;
  const int p = (int)(i % hw);
  const long nc = i / hw;
  const int ch = (int)(nc % c);
  const long n = nc / c;
  y[i] = x[(n * hw + p) * cp + ch];
}

// [o][c][khw] -> [o][khw][cp], zero in the pad channels
template <typename T>
__global__ __launch_bounds__(256) void repack_weights_kernel(const T* __restrict__ w, T* __restrict__ y,
                                                             long total, int c, int khw, int cp) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int ch = (int)(i % cp);
  const long ot = i / cp;
  const int tpos = (int)(ot % khw);
  const long o = ot / khw;
  T v = (T)0.0f;
  if (ch < c) v = w[(o * c + ch) * khw + tpos];
  y[i] = v;
}

// [o][9][cp] -> the order in which the independent-wavefront 3x3 kernel's lanes fetch their MFMA
// operands: [filter tile of 16][64-byte channel chunk][tap][lane = quad * 16 + filter][16 bytes], so
// that one wavefront-wide load reads 1 KiB of consecutive memory; zero past the last filter / channel
template <typename T>
__global__ __launch_bounds__(256) void repack_wave_kernel(const T* __restrict__ w, T* __restrict__ y, long total,
                                                          int o_count, int cp, int nchunk) {
  constexpr int EPI = 16 / (int)sizeof(T);
  const long i = (long)blockIdx.x * 256 + threadIdx.x;   // one element of the output
  if (i >= total) return;
  const int e = (int)(i % EPI);
  long q = i / EPI;
  const int lane = (int)(q & 63); q >>= 6;
  const int tap = (int)(q % 9); q /= 9;
  const int chunk = (int)(q % nchunk);
  const long tm = q / nchunk;
  const long o = tm * 16 + (lane & 15);
  const int ch = chunk * 4 * EPI + (lane >> 4) * EPI + e;
  T v = (T)0.0f;
  if (o < o_count && ch < cp) v = w[(o * 9 + tap) * cp + ch];
  y[i] = v;
}

// [rows][k] (k contiguous) -> the order in which the reduction-split kernel's lanes fetch their MFMA
// operands: [16-row tile][64-byte round of k][lane = quad * 16 + row][16 bytes]; zero past the last row / k
template <typename T>
__global__ __launch_bounds__(256) void repack_rows_kernel(const T* __restrict__ w, T* __restrict__ y, long total,
                                                          int rows, int k, int rounds) {
  constexpr int EPI = 16 / (int)sizeof(T);
  const long i = (long)blockIdx.x * 256 + threadIdx.x;   // one element of the output
  if (i >= total) return;
  const int e = (int)(i % EPI);
  long q = i / EPI;
  const int lane = (int)(q & 63); q >>= 6;
  const int rnd = (int)(q % rounds);
  const long tm = q / rounds;
  const long row = tm * 16 + (lane & 15);
  const int kk = rnd * 4 * EPI + (lane >> 4) * EPI + e;
  T v = (T)0.0f;
  if (row < rows && kk < k) v = w[row * k + kk];
  y[i] = v;
}

// Every input pixel of a 2x2 map lies inside the 3x3 window (pad 1) of every output pixel, so
// the layer is one dense matrix from the whole input map to the whole output map: the tap that
// links input pixel (iy, ix) to output pixel (oy, ox) is (iy - oy + 1, ix - ox + 1).
template <typename T>
__global__ __launch_bounds__(256) void repack_map2x2_kernel(const T* __restrict__ w, const float* __restrict__ bias,
                                                            T* __restrict__ y, float* __restrict__ bias_out, int o_count,
                                                            int c, int cp_in, int cp_out, int rows_by_channel) {
  const long total = (long)16 * cp_out * cp_in;
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int col = (int)(i % (4 * cp_in));
  const int row = (int)(i / (4 * cp_in));
  const int pi = col / cp_in, ch = col % cp_in;
  const int po = rows_by_channel ? (row & 3) : row / cp_out;
  const int o = rows_by_channel ? (row >> 2) : row % cp_out;
  T v = (T)0.0f;
  if (o < o_count && ch < c) {
    const int u = (pi >> 1) - (po >> 1) + 1, t = (pi & 1) - (po & 1) + 1;
    v = w[((long)o * c + ch) * 9 + u * 3 + t];
  }
  y[i] = v;
  if (col == 0) bias_out[row] = (bias && o < o_count) ? bias[o] : 0.0f;
}

// [o][ktot] -> [rows][kp], zero beyond ktot and beyond the last filter
template <typename T>
__global__ __launch_bounds__(256) void repack_stem_kernel(const T* __restrict__ w, T* __restrict__ y, long total,
                                                          int o_count, int ktot, int kp) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int k = (int)(i % kp);
  const long o = i / kp;
  T v = (T)0.0f;
  if (o < o_count && k < ktot) v = w[o * ktot + k];
  y[i] = v;
}

// OIHW 7x7 weights -> [rows][224]: k = u * 32 + (v + 1) * 4 + c (window row, window column shifted by one slot,
// channel), zero elsewhere
template <typename T>
__global__ __launch_bounds__(256) void repack_stem7_kernel(const T* __restrict__ w, T* __restrict__ y, long total,
                                                           int o_count, int c_count) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int k = (int)(i % kStem7K);
  const long o = i / kStem7K;
  const int u = k >> 5, slot = (k >> 2) & 7, c = k & 3;
  T v = (T)0.0f;
  if (o < o_count && c < c_count && slot >= 1) v = w[((o * c_count + c) * 7 + u) * 7 + (slot - 1)];
  y[i] = v;
}

inline dim3 blocks_for(long total) { return dim3((unsigned)((total + 255) / 256)); }

int plane_slices(int total) {
  int s = (total + 1023) / 1024;
  return s < 1 ? 1 : (s > 64 ? 64 : s);
}

template <typename T>
int depthwise_dispatch(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                       const void* res, void* y, hipStream_t s) {
  const int ho = conv_out_dim(d.h, d.kh, d.stride, d.pad), wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  dim3 grid((unsigned)(d.n * d.c_in), (unsigned)plane_slices(ho * wo));
#define GO(K)                                                                                     \
  hipLaunchKernelGGL((depthwise_kernel<T, K>), grid, dim3(256), 0, s, (const T*)x, (const T*)w,  \
                     bias, (const T*)res, (T*)y, d.c_in, d.h, d.w, ho, wo, d.stride, d.pad, d.act)
  switch (d.kh) {
    case 1: GO(1); break;
    case 3: GO(3); break;
    case 5: GO(5); break;
    case 7: GO(7); break;
    default: return CPRUNE_ERR_UNSUPPORTED;
  }
#undef GO
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

}  // namespace

int launch_conv_depthwise(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                          const void* residual, void* y, hipStream_t s) {
  if (d.kh != d.kw) return CPRUNE_ERR_UNSUPPORTED;
  if (d.dtype == CPRUNE_F32) return depthwise_dispatch<float>(d, x, w, bias, residual, y, s);
  if (d.dtype == CPRUNE_F16) return depthwise_dispatch<_Float16>(d, x, w, bias, residual, y, s);
  return depthwise_dispatch<__bf16>(d, x, w, bias, residual, y, s);
}

int launch_maxpool(const void* x, int n, int c, int h, int w, int k, int stride, int pad, int dt,
                   void* y, hipStream_t s) {
  const int ho = conv_out_dim(h, k, stride, pad), wo = conv_out_dim(w, k, stride, pad);
  dim3 grid((unsigned)(n * c), (unsigned)plane_slices(ho * wo));
  if (dt == CPRUNE_F32)
    hipLaunchKernelGGL(maxpool_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (float*)y, h, w,
                       ho, wo, k, stride, pad);
  else if (dt == CPRUNE_F16)
    hipLaunchKernelGGL(maxpool_kernel<_Float16>, grid, dim3(256), 0, s, (const _Float16*)x,
                       (_Float16*)y, h, w, ho, wo, k, stride, pad);
  else
    hipLaunchKernelGGL(maxpool_kernel<__bf16>, grid, dim3(256), 0, s, (const __bf16*)x, (__bf16*)y, h,
                       w, ho, wo, k, stride, pad);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int launch_gavgpool(const void* x, int n, int c, int hw, int dt, void* y, hipStream_t s) {
  const int planes = n * c;
  dim3 grid((unsigned)((planes + 3) / 4));
  if (dt == CPRUNE_F32)
    hipLaunchKernelGGL(gavgpool_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (float*)y,
                       planes, hw);
  else if (dt == CPRUNE_F16)
    hipLaunchKernelGGL(gavgpool_kernel<_Float16>, grid, dim3(256), 0, s, (const _Float16*)x,
                       (_Float16*)y, planes, hw);
  else
    hipLaunchKernelGGL(gavgpool_kernel<__bf16>, grid, dim3(256), 0, s, (const __bf16*)x, (__bf16*)y,
                       planes, hw);
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

#define CPRUNE_BY_DTYPE(DT, CALL)                      \
  do {                                                  \
    if ((DT) == CPRUNE_F32) { typedef float T; CALL; }  \
    else if ((DT) == CPRUNE_F16) { typedef _Float16 T; CALL; } \
    else { typedef __bf16 T; CALL; }                    \
  } while (0)

int launch_maxpool_nhwc(const void* x, int n, int cp, int h, int w, int k, int stride, int pad, int dt,
                        void* y, hipStream_t s) {
  const int ho = conv_out_dim(h, k, stride, pad), wo = conv_out_dim(w, k, stride, pad);
  const long total = (long)n * ho * wo * cp;
  const int vec = dt == CPRUNE_F32 ? 4 : 8;
  if (cp % vec == 0 && total / vec < (1L << 32)) {
    const long tv = total / vec;
    CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(maxpool_nhwc_vec_kernel<T>, blocks_for(tv), dim3(256), 0, s, (const T*)x,
                                           (T*)y, (unsigned)tv, cp, h, w, ho, wo, k, stride, pad));
    CPRUNE_LAUNCH_CHECK();
    return CPRUNE_OK;
  }
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(maxpool_nhwc_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)x,
                                         (T*)y, total, cp, h, w, ho, wo, k, stride, pad));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int launch_gavgpool_nhwc(const void* x, int n, int cp, int hw, int dt, void* y, hipStream_t s) {
  const int total = n * cp;
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(gavgpool_nhwc_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)x,
                                         (T*)y, total, cp, hw));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

template <typename T>
static int depthwise_nhwc_dispatch(const cprune_conv_desc& d, int cp, const void* x, const void* w,
                                   const float* bias, const void* res, void* y, hipStream_t s) {
  const int ho = conv_out_dim(d.h, d.kh, d.stride, d.pad), wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  constexpr int V = VecOf<T>::V;
  // vectorised kernel: 3x3 and 5x5 at stride 1 or 2, channel stride a whole number of vectors;
  // four outputs per thread when that still leaves every compute unit several work-groups
  if ((d.kh == 3 || d.kh == 5) && (d.stride == 1 || d.stride == 2) && cp % V == 0) {
    const long per_row = (long)d.n * ho * (cp / V);
    const int tx = per_row * ((wo + 3) / 4) >= 256L * 1024 ? 4 : 1;
    const int xblocks = (wo + tx - 1) / tx;
    const long total = per_row * xblocks;
    if (total < (1L << 32)) {
#define GOV(K, S, TX)                                                                                           \
      hipLaunchKernelGGL((depthwise_nhwc_vec_kernel<T, K, S, TX>), blocks_for(total), dim3(256), 0, s, (const T*)x, \
                         (const T*)w, bias, (const T*)res, (T*)y, (unsigned)total, d.c_in, cp, d.h, d.w, ho, wo,  \
                         xblocks, d.pad, d.act)
      const int key = d.kh * 100 + d.stride * 10 + tx;
      switch (key) {
        case 311: GOV(3, 1, 1); break;
        case 314: GOV(3, 1, 4); break;
        case 321: GOV(3, 2, 1); break;
        case 324: GOV(3, 2, 4); break;
        case 511: GOV(5, 1, 1); break;
        case 514: GOV(5, 1, 4); break;
        case 521: GOV(5, 2, 1); break;
        case 524: GOV(5, 2, 4); break;
      }
#undef GOV
      CPRUNE_LAUNCH_CHECK();
      return CPRUNE_OK;
    }
  }
  const long total = (long)d.n * ho * wo * cp;
#define GO(K)                                                                                          \
  hipLaunchKernelGGL((depthwise_nhwc_kernel<T, K>), blocks_for(total), dim3(256), 0, s, (const T*)x,   \
                     (const T*)w, bias, (const T*)res, (T*)y, total, d.c_in, cp, d.h, d.w, ho, wo,     \
                     d.stride, d.pad, d.act)
  switch (d.kh) {
    case 1: GO(1); break;
    case 3: GO(3); break;
    case 5: GO(5); break;
    case 7: GO(7); break;
    default: return CPRUNE_ERR_UNSUPPORTED;
  }
#undef GO
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int launch_depthwise_nhwc(const cprune_conv_desc& d, int cp, const void* x, const void* w, const float* bias,
                          const void* residual, void* y, hipStream_t s) {
  if (d.kh != d.kw) return CPRUNE_ERR_UNSUPPORTED;
  if (d.dtype == CPRUNE_F32) return depthwise_nhwc_dispatch<float>(d, cp, x, w, bias, residual, y, s);
  if (d.dtype == CPRUNE_F16) return depthwise_nhwc_dispatch<_Float16>(d, cp, x, w, bias, residual, y, s);
  return depthwise_nhwc_dispatch<__bf16>(d, cp, x, w, bias, residual, y, s);
}

int launch_nchw_to_nhwc(const void* x, int n, int c, int hw, int cp, int dt, void* y, hipStream_t s) {
  const long total = (long)n * hw * cp;
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(nchw_to_nhwc_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)x,
                                         (T*)y, total, c, hw, cp));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int launch_nhwc_to_nchw(const void* x, int n, int c, int hw, int cp, int dt, void* y, hipStream_t s) {
  const long total = (long)n * c * hw;
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(nhwc_to_nchw_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)x,
                                         (T*)y, total, c, hw, cp));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int launch_repack_weights(const void* w, int o, int c, int khw, int cp, int dt, void* y, hipStream_t s) {
  const long total = (long)o * khw * cp;
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(repack_weights_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)w,
                                         (T*)y, total, c, khw, cp));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

size_t wave_packed_bytes(int o, int cp, int dt) {
  const int cc = dt == CPRUNE_F32 ? 16 : 32;   // channels per 64-byte chunk
  return (size_t)((o + 15) / 16) * ((cp + cc - 1) / cc) * 9 * 1024;
}

int launch_repack_wave(const void* w_khwc, int o, int cp, int dt, void* y, hipStream_t s) {
  const int cc = dt == CPRUNE_F32 ? 16 : 32;
  const int nchunk = (cp + cc - 1) / cc;
  const long total = (long)(wave_packed_bytes(o, cp, dt) / dtype_size(dt));
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(repack_wave_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)w_khwc,
                                         (T*)y, total, o, cp, nchunk));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

size_t rows_packed_bytes(int rows, int k, int dt) {
  const size_t per_round = 64 / dtype_size(dt);
  return (size_t)((rows + 15) / 16) * ((k + per_round - 1) / per_round) * 1024;
}

int launch_repack_rows(const void* w, int rows, int k, int dt, void* y, hipStream_t s) {
  const int per_round = (int)(64 / dtype_size(dt));
  const int rounds = (k + per_round - 1) / per_round;
  const long total = (long)(rows_packed_bytes(rows, k, dt) / dtype_size(dt));
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(repack_rows_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)w, (T*)y,
                                         total, rows, k, rounds));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int stem_packed_k(int k, int dt) {
  const int rk = dt == CPRUNE_F32 ? 16 : 32;   // k per 64-byte MFMA round
  return (3 * k * k + rk - 1) / rk * rk;
}

int launch_repack_stem(const void* w, int o, int ktot, int rows, int kp, int dt, void* y, hipStream_t s) {
  const long total = (long)rows * kp;
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(repack_stem_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)w, (T*)y,
                                         total, o, ktot, kp));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int launch_repack_stem7(const void* w, int o, int c, int rows, int dt, void* y, hipStream_t s) {
  const long total = (long)rows * kStem7K;
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(repack_stem7_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)w, (T*)y,
                                         total, o, c));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

int launch_repack_map2x2(const void* w, const float* bias, int o, int c, int cp_in, int cp_out,
                         int rows_by_channel, int dt, void* w_out, float* bias_out, hipStream_t s) {
  const long total = (long)16 * cp_out * cp_in;
  CPRUNE_BY_DTYPE(dt, hipLaunchKernelGGL(repack_map2x2_kernel<T>, blocks_for(total), dim3(256), 0, s, (const T*)w, bias,
                                         (T*)w_out, bias_out, o, c, cp_in, cp_out, rows_by_channel));
  CPRUNE_LAUNCH_CHECK();
  return CPRUNE_OK;
}

}  // namespace cprune
