// 1x1 / stride 1 convolution with a SHORT reduction, channels-last: the expansion layers of
// inverted-residual blocks (16-96 input channels, several times as many filters, large maps).
// Such a layer is a plain matrix product Y[p][o] = sum_k X[p][k] W[o][k] that moves far more
// bytes than it multiplies: the tiled kernels spend their time on per-tile set-up (im2col
// bookkeeping a 1x1 window does not need), not on the two or three reduction slabs.
//
// Here a work-group is persistent: it stages its filter tile (at most 128 filters, the whole
// reduction) in LDS once and then streams 64-pixel tiles through it.  A pixel's input row is
// k-contiguous, so a lane's B operand for a 64-byte round is one 16-byte global load (no
// staging, every byte of X read once per filter tile); the next tile's operands are in flight
// while this one is multiplied.  Output stores are 16 bytes per lane, 64 contiguous bytes per
// pixel and filter block.  Bound: HBM (X once per filter tile + Y once).
//
// Same MFMA blocks, lane layout and k-permutation as the other dense kernels.
#pragma once
#include "conv_nhwc_kernel.hpp"

namespace cprune {

template <typename T, int MB, int NR>
__global__ __launch_bounds__(256) void conv_pw_kernel(ConvArgs a) {
  constexpr int NT = 256;
  constexpr int ES = (int)sizeof(T);
  constexpr int MT = MB * 16;
  constexpr int AROW = NR * 64 + 16;
  constexpr int U = 4;

  extern __shared__ __attribute__((aligned(16))) unsigned char sA[];   // [MT][AROW] filter tile, whole reduction

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int r = lane & 15, g4 = lane >> 4;

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t wr = make_rsrc(a.w, a.w_bytes);
  const unsigned row_bytes = (unsigned)a.K * ES;       // a multiple of 16: channel strides are whole vectors
  const int o0 = blockIdx.y * MT;

  // ---- once: the filter tile (rows past the last filter and bytes past the reduction read as zero) ----
  for (int b0 = t; b0 < MT * NR * 4; b0 += NT * U) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = b0 + u * NT;
      const int m = idx / (NR * 4), q = idx - m * (NR * 4);
      const bool ok = idx < MT * NR * 4 && o0 + m < a.O && (unsigned)q * 16 < row_bytes;
      v[u] = load_b128(wr, ok ? (unsigned)(o0 + m) * row_bytes + q * 16 : kOutOfRange, 0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = b0 + u * NT;
      if (idx < MT * NR * 4) {
        const int m = idx / (NR * 4), q = idx - m * (NR * 4);
        *(uint4*)&sA[m * AROW + q * 16] = v[u];
      }
    }
  }

  int mb_count = (a.O - o0 + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;
  const int a_frag = r * AROW + g4 * 16;

  int worker;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    worker = xcd * q + (xcd < rem ? xcd : rem) + local;
  }

  // operands of a pixel tile: lane (r, g4) takes bytes [64 rnd + 16 g4, +16) of pixel tile * 64 + 16 wave + r
  uint4 bf[NR], nf[NR];
  auto fetch = [&](int tile, uint4 (&f)[NR]) {
    const int p = tile * 64 + wave * 16 + r;
#pragma unroll
    for (int rnd = 0; rnd < NR; ++rnd) {
      const unsigned off = (unsigned)rnd * 64 + g4 * 16;
      f[rnd] = load_b128(xr, (p < a.P && off < row_bytes) ? (unsigned)p * row_bytes + off : kOutOfRange, 0);
    }
  };
  if (worker < a.tiles_p) fetch(worker, nf);
  __syncthreads();                 // the filter tile is in LDS

  for (int tile = worker; tile < a.tiles_p; tile += (int)gridDim.x) {
#pragma unroll
    for (int rnd = 0; rnd < NR; ++rnd) bf[rnd] = nf[rnd];
    if (tile + (int)gridDim.x < a.tiles_p) fetch(tile + (int)gridDim.x, nf);

    float4_t acc[MB][1];
#pragma unroll
    for (int i = 0; i < MB; ++i) acc[i][0] = (float4_t){0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](auto mbc_tag) {
      constexpr int MBC = decltype(mbc_tag)::value;
#pragma unroll
      for (int rnd = 0; rnd < NR; ++rnd) {
        uint4 af[MB], b1[1];
        b1[0] = bf[rnd];
#pragma unroll
        for (int i = 0; i < MBC; ++i) af[i] = *(const uint4*)&sA[a_frag + i * 16 * AROW + rnd * 64];
        mma_slab<T, MBC, 1, MB>(af, b1, acc);
      }
    };
    switch (mb_count) {
#define CPRUNE_MBC_CASE(V) \
  case V: if constexpr (MB >= V) multiply(std::integral_constant<int, V>{}); break;
      CPRUNE_MBC_CASE(1) CPRUNE_MBC_CASE(2) CPRUNE_MBC_CASE(3) CPRUNE_MBC_CASE(4)
      CPRUNE_MBC_CASE(5) CPRUNE_MBC_CASE(6) CPRUNE_MBC_CASE(7) CPRUNE_MBC_CASE(8)
#undef CPRUNE_MBC_CASE
      default: break;
    }

    const int p = tile * 64 + wave * 16 + r;
    if (p < a.P) {
#pragma unroll
      for (int i = 0; i < MB; ++i) nhwc_store4<T>(a, acc[i][0], p, o0 + i * 16 + 4 * g4);
    }
  }
}

// Variants: id, mb (16-filter blocks per tile), nr (64-byte rounds of the reduction the tile holds)
#define CPRUNE_PW_LIST(X) \
  X(0, 2, 1) X(1, 2, 2) X(2, 2, 3) X(3, 2, 4) X(4, 2, 6)    \
  X(5, 4, 1) X(6, 4, 2) X(7, 4, 3) X(8, 4, 4) X(9, 4, 6)    \
  X(10, 8, 1) X(11, 8, 2) X(12, 8, 3) X(13, 8, 4) X(14, 8, 6)

constexpr int kNumPw = 15;

template <typename T>
inline void launch_pw(int id, dim3 grid, hipStream_t s, const ConvArgs& a) {
#define CPRUNE_PW_CASE(ID, MB_, NR_)                                                                             \
  case ID:                                                                                                       \
    hipLaunchKernelGGL((conv_pw_kernel<T, MB_, NR_>), grid, dim3(256), (size_t)(MB_ * 16) * (NR_ * 64 + 16), s, a); \
    break;
  switch (id) { CPRUNE_PW_LIST(CPRUNE_PW_CASE) }
#undef CPRUNE_PW_CASE
}

void launch_conv_pw_f32(int id, dim3 grid, hipStream_t s, const ConvArgs& a);
void launch_conv_pw_f16(int id, dim3 grid, hipStream_t s, const ConvArgs& a);
void launch_conv_pw_bf16(int id, dim3 grid, hipStream_t s, const ConvArgs& a);

}  // namespace cprune
