// The first two layers of a network in one kernel, where both are 3x3 / stride 1 / pad 1
// convolutions and the first has at most 32 filters (the opening of a VGG-style network:
// image -> conv -> conv [-> 2x2 pool]).  The first layer's output is the largest activation of
// such a network and is read only by the second layer; here it never leaves the compute unit.
//
// A work-group owns an 8 x 16 tile of the second layer's output pixels and 16 * MB of its
// filters.  Stage 1: the 12 x 20 patch of the image (all channels) goes to LDS and the first
// layer is computed on the 10 x 18 pixels the second layer's taps touch (its whole reduction,
// c_in * 9 <= 27 terms, is one or two MFMA rounds; the im2col operand is gathered from the
// patch through a table of offsets, as in the first-layer kernel); bias and activation are
// applied, pixels outside the image become the second layer's zero padding, and the result is
// written to LDS channels-last, which is exactly the input patch of the spatial-patch kernel.
// Stage 2: that kernel's multiply, all of the (at most 32) input channels in one chunk, with the
// second layer's weight tile in flight while stage 1 runs; then its epilogue (bias, activation,
// optional fused 2x2 max-pool).  The halo costs stage 1 40 % more pixels than the tile has, of a
// layer that is a few percent of the second layer's work.
//
// Same MFMA blocks, lane layout and k-permutation as the other dense kernels.
#pragma once
#include <atomic>
#include "conv_patch_kernel.hpp"

namespace cprune {

struct Stem2Args {
  const void* x;        // [n][c][h][w] image, c <= 3
  const void* w1;       // [32][kp] first-layer weights packed by launch_repack_stem (k = (c, u, v), zero padded)
  const float* b1;      // [c1] or null
  int C, C1, Cp1;       // image channels; first-layer filters (<= 32) and their channel stride in w2 (<= 32)
  int act1;
  PatchArgs p;          // the second layer as the spatial-patch kernel sees it (x unused; w = [c2][9][cp1];
                        // tiles_n = images, tiles_y / tiles_x of 8 x 16 pixels, tiles_m of 16 * MB filters)
};

template <typename T, int MB>
__global__ __launch_bounds__(256) void conv_stem2_kernel(Stem2Args a) {
  constexpr int NT = 256;
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;                 // elements per 16-byte quad
  constexpr int RK = 4 * EPI;                  // k (or channels) per 64-byte MFMA round
  constexpr int TH = 8, TW = 16, NB = 2;       // second layer: 128 pixels, wave w owns rows 2w, 2w + 1
  constexpr int MT = MB * 16;
  constexpr int CMAX = 3, C1MAX = 32;
  constexpr int XH = TH + 4, XW = TW + 4, XWP = XW;           // image patch
  constexpr int PH = TH + 2, PW = TW + 2, NPATCH = PH * PW;   // first-layer pixels = second layer's patch
  constexpr int KP = (CMAX * 9 + RK - 1) / RK * RK;           // first-layer reduction padded to whole rounds
  constexpr int NR1 = KP / RK;
  constexpr int AROW1 = KP * ES + 16;
  constexpr int KQ = C1MAX * ES / 64;                         // 64-byte rounds per tap of the second layer
  constexpr int BROW = 64 * KQ + 16;
  constexpr int AROW2 = 9 * 64 * KQ + 16;
  constexpr int NQ = 4 * KQ;
  constexpr int NBLK1 = (NPATCH + 15) / 16;                   // 16-pixel blocks of stage 1
  constexpr int NIA = (MT * 9 * NQ + NT - 1) / NT;

  // dynamic LDS: first-layer weights, offset table, image patch, second layer's patch and weight tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* const sW1 = smem;
  int* const sT = (int*)(sW1 + C1MAX * AROW1);
  T* const sX = (T*)((unsigned char*)sT + KP * 4);
  unsigned char* const sB = (unsigned char*)sX + (CMAX * XH * XWP * ES + 15) / 16 * 16;
  unsigned char* const sA = sB + NPATCH * BROW;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int r = lane & 15, g4 = lane >> 4;
  const PatchArgs& p = a.p;

  int tile;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    tile = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  // filter tiles fastest (the image is the larger operand)
  const int rest0 = (int)fast_div((unsigned)tile, p.magic_m);
  const int tile_m = tile - rest0 * p.tiles_m;
  const int q_x = (int)fast_div((unsigned)rest0, p.magic_x);
  const int n = (int)fast_div((unsigned)q_x, p.magic_y);
  const int tx0 = (rest0 - q_x * p.tiles_x) * TW;
  const int ty0 = (q_x - n * p.tiles_y) * TH;
  const int o0 = tile_m * MT;

  // ---- second layer's weight tile: requested first, stored behind stage 1 ----
  const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.w, p.w_bytes);
  uint4 areg[NIA];
  int a_lds[NIA];
#pragma unroll
  for (int j = 0; j < NIA; ++j) {
    const int idx = t + NT * j;
    const int q = idx % NQ;
    const int tap = (idx / NQ) % 9;
    const int m = (idx / NQ) / 9;
    const bool item = m < MT;
    const int o = o0 + m;
    const unsigned off = (item && o < p.O && q * EPI < a.Cp1) ? (unsigned)((o * 9 + tap) * a.Cp1 + q * EPI) * ES : kOutOfRange;
    areg[j] = load_b128(wr, off, 0);      // zeros past the last filter and channel
    a_lds[j] = item ? m * AROW2 + tap * (64 * KQ) + q * 16 : MT * AROW2 - 16;
  }

  // ---- stage 1 staging: offset table, first-layer weights, image patch ----
  const int ktot = a.C * 9;
  for (int k = t; k < KP; k += NT) {
    int off = 0;
    if (k < ktot) {
      const int c = k / 9, uv = k - c * 9;
      const int u = uv / 3, v = uv - u * 3;
      off = (c * XH + u) * XWP + v;
    }
    sT[k] = off;
  }
  {
    constexpr int QROW = KP * ES / 16;
    const uint4* __restrict__ wq = (const uint4*)a.w1;
    for (int idx = t; idx < C1MAX * QROW; idx += NT) {
      const int m = idx / QROW, q = idx - m * QROW;
      *(uint4*)&sW1[m * AROW1 + q * 16] = wq[idx];
    }
  }
  {
    const T* __restrict__ xg = (const T*)a.x;
    const int iy0 = ty0 - 2, ix0 = tx0 - 2;
    for (int idx = t; idx < CMAX * XH * XWP; idx += NT) {
      const int px = idx % XWP;
      const int cy = idx / XWP;
      const int py = cy % XH, c = cy / XH;
      const int iy = iy0 + py, ix = ix0 + px;
      T val = (T)0.0f;
      if (c < a.C && n < p.N && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W)
        val = xg[((size_t)(n * a.C + c) * p.H + iy) * p.W + ix];
      sX[idx] = val;
    }
  }
  __syncthreads();

  // ---- stage 1: the first layer on the 10 x 18 patch, 16 pixels x 32 filters at a time ----
  float4_t bias1[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) bias1[i] = load_bias4(a.b1, a.C1, i * 16 + 4 * g4);
  for (int blk = wave; blk < NBLK1; blk += 4) {
    const int pp = blk * 16 + r;
    const int ppc = pp < NPATCH ? pp : NPATCH - 1;      // lanes past the patch recompute its last pixel (not stored)
    const int py = ppc / PW, px = ppc - py * PW;
    const int pbase = py * XWP + px;
    float4_t acc1[2][1];
    acc1[0][0] = (float4_t){0.f, 0.f, 0.f, 0.f};
    acc1[1][0] = (float4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rnd = 0; rnd < NR1; ++rnd) {
      int offs[EPI];
#pragma unroll
      for (int q = 0; q < EPI / 4; ++q) {
        const int4 o4 = *(const int4*)&sT[rnd * RK + g4 * EPI + 4 * q];
        offs[4 * q] = o4.x; offs[4 * q + 1] = o4.y; offs[4 * q + 2] = o4.z; offs[4 * q + 3] = o4.w;
      }
      uint4 af[2], bf[1];
#pragma unroll
      for (int i = 0; i < 2; ++i) af[i] = *(const uint4*)&sW1[(i * 16 + r) * AROW1 + rnd * 64 + g4 * 16];
      T* be = reinterpret_cast<T*>(&bf[0]);
#pragma unroll
      for (int e2 = 0; e2 < EPI; ++e2) be[e2] = sX[pbase + offs[e2]];
      mma_slab<T, 2, 1, 2>(af, bf, acc1);
    }
    // lane: filters 16 i + 4 g4 .. + 3 of pixel pp.  Outside the image the second layer sees zero padding.
    const int iy = ty0 - 1 + py, ix = tx0 - 1 + px;
    const bool inside = (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
    if (pp < NPATCH) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int ch = i * 16 + 4 * g4;
        const float4_t b = bias1[i];
        alignas(16) T out[4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
          out[v] = Elem<T>::from_f32(inside ? apply_act(acc1[i][0][v] + b[v], a.act1) : 0.0f);
        if constexpr (ES == 4) *(uint4*)&sB[pp * BROW + ch * ES] = *reinterpret_cast<const uint4*>(out);
        else *(uint2*)&sB[pp * BROW + ch * ES] = *reinterpret_cast<const uint2*>(out);
      }
    }
  }
  // the second layer's weight tile, in flight since the start
#pragma unroll
  for (int j = 0; j < NIA; ++j) *(uint4*)&sA[a_lds[j]] = areg[j];
  __syncthreads();

  // ---- stage 2: the second layer, every input channel in one chunk ----
  float4_t bias4[MB];    // for the epilogue, requested ahead of the multiply
  load_tile_bias<T, MB>(p, o0, g4, bias4);
  int b_frag[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int id = wave * (NB * 16) + j * 16 + r;
    b_frag[j] = ((id / TW) * PW + id % TW) * BROW + g4 * 16;
  }
  const int a_frag = r * AROW2 + g4 * 16;
  float4_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};
  int mb_count = (p.O - o0 + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;
  auto multiply = [&](auto mbc_tag) {
    constexpr int MBC = decltype(mbc_tag)::value;
    constexpr int NR = 9 * KQ;
    uint4 af[2][MB], bf[2][NB];
    auto fetch = [&](int rnd, uint4 (&fa)[MB], uint4 (&fb)[NB]) {
      const int tap = rnd / KQ, q4 = rnd % KQ;
      const int boff = ((tap / 3) * PW + (tap % 3)) * BROW + q4 * 64;
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[j] = *(const uint4*)&sB[b_frag[j] + boff];
#pragma unroll
      for (int i = 0; i < MBC; ++i) fa[i] = *(const uint4*)&sA[a_frag + i * 16 * AROW2 + tap * (64 * KQ) + q4 * 64];
    };
    fetch(0, af[0], bf[0]);
#pragma unroll
    for (int rnd = 0; rnd < NR; ++rnd) {
      if (rnd + 1 < NR) fetch(rnd + 1, af[(rnd + 1) & 1], bf[(rnd + 1) & 1]);
      __builtin_amdgcn_s_setprio(1);
      mma_slab<T, MBC, NB, MB>(af[rnd & 1], bf[rnd & 1], acc);
      __builtin_amdgcn_s_setprio(0);
    }
  };
  switch (mb_count) {
    case 1: multiply(std::integral_constant<int, 1>{}); break;
    case 2: if constexpr (MB >= 2) multiply(std::integral_constant<int, 2>{}); break;
    case 3: if constexpr (MB >= 3) multiply(std::integral_constant<int, 3>{}); break;
    case 4: if constexpr (MB >= 4) multiply(std::integral_constant<int, 4>{}); break;
    default: break;
  }

  patch_epilogue<T, MB, TH, TW, NB>(p, acc, wave, r, g4, n, ty0, tx0, o0, bias4);
}

// LDS bytes of the kernel for a filter tile of mb blocks and an element size
constexpr size_t stem2_lds_bytes(int mb, int es) {
  const int rk = 64 / es, kp = (27 + rk - 1) / rk * rk, kq = 32 * es / 64;
  return (size_t)32 * (kp * es + 16) + (size_t)kp * 4 + (size_t)(3 * 12 * 20 * es + 15) / 16 * 16 +
         (size_t)180 * (64 * kq + 16) + (size_t)mb * 16 * (9 * 64 * kq + 16);
}

// mb in {1, 2, 4} (16-filter blocks of the second layer per tile); grid = images x 8x16 pixel tiles x filter tiles
template <typename T>
inline int launch_stem2(int mb, dim3 grid, hipStream_t s, const Stem2Args& a) {
#define CPRUNE_STEM2(MB_)                                                                            \
  if (mb == MB_) {                                                                                   \
    constexpr size_t lds = stem2_lds_bytes(MB_, (int)sizeof(T));                                     \
    static_assert(lds <= 160 * 1024, "LDS budget");                                                  \
    static std::atomic<bool> raised{false};   /* more than the default 64 KiB has to be asked for */ \
    if (lds > 65536 && !raised.load(std::memory_order_relaxed)) {                                    \
      CPRUNE_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_stem2_kernel<T, MB_>),  \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));     \
      raised.store(true, std::memory_order_relaxed);                                                 \
    }                                                                                                \
    hipLaunchKernelGGL((conv_stem2_kernel<T, MB_>), grid, dim3(256), lds, s, a);                     \
    return CPRUNE_OK;                                                                                \
  }
  CPRUNE_STEM2(1) CPRUNE_STEM2(2) CPRUNE_STEM2(4)
#undef CPRUNE_STEM2
  return CPRUNE_ERR_UNSUPPORTED;
}

int launch_conv_stem2_f32(int mb, dim3 grid, hipStream_t s, const Stem2Args& a);
int launch_conv_stem2_f16(int mb, dim3 grid, hipStream_t s, const Stem2Args& a);
int launch_conv_stem2_bf16(int mb, dim3 grid, hipStream_t s, const Stem2Args& a);

}  // namespace cprune
