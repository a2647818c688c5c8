// 3x3 / stride 1 / pad 1 convolution, channels-last, spatial patch staged once per
// channel chunk (as conv_patch_kernel), on 32x32 MFMA blocks, with the option of
// splitting the reduction between the wavefronts of a work-group.
//
// Why a second kernel.  One wavefront alone on its SIMD issues the 16x16x4 fp32
// MFMA at about three quarters of the pipe's rate (measured: 120 of 157 TFLOP/s with one
// wavefront per SIMD, 141 with eight), the 32x32x2 form at 97 %.  Layers whose grids
// leave a compute unit one work-group (small maps, deep channels: the second half of
// VGG-16) are bound by exactly that.  A 32x32 block is four times coarser, so on such
// layers there are too few blocks to give every wavefront its own: here WK = 4 / WPX
// wavefronts share one block column and split each chunk's rounds between them (every
// staged element is then read from LDS by exactly one wavefront instead of by all
// four); their partial sums meet in LDS once, at the end of the tile.
//
// Lane layout of v_mfma_f32_32x32x2_f32 (and the x16 16-bit forms): lane l feeds row /
// column l % 32 with k-slot l / 32; it ends up with 16 results, register v holding row
// 8 * (v / 4) + 4 * (l / 32) + v % 4 of column l % 32.  Inside a 64-byte round of k
// lane half h = l / 32 takes bytes 32h .. 32h + 31 of both operands (fp32: eight MFMAs,
// one per float; 16-bit: two MFMAs, one per 16-byte quad).
#pragma once
#include "conv_patch_kernel.hpp"

namespace cprune {

typedef float float16_t __attribute__((ext_vector_type(16)));

template <typename T, int MB2, int NB2, int WPX, int TH, int TW, int NI, int KQ>
__global__ __launch_bounds__(256) void conv_patch32_kernel(PatchArgs a) {
  constexpr int NT = 256;
  constexpr int WK = 4 / WPX;             // wavefronts that split the rounds of one block column
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;
  constexpr int CC = 4 * EPI * KQ;
  constexpr int NQ = 4 * KQ;
  constexpr int PT = TH * TW * NI;
  constexpr int MT = MB2 * 32;
  constexpr int PW = TW + 2, PH = TH + 2;
  constexpr int NPATCH = NI * PH * PW;
  constexpr int BROW = 64 * KQ + 16;
  constexpr int AROW = 9 * 64 * KQ + 16;
  constexpr int NIB = (NPATCH * NQ + NT - 1) / NT;
  constexpr int NIA = (MT * 9 * NQ + NT - 1) / NT;
  constexpr int NR = 9 * KQ;              // rounds per chunk
  static_assert(WPX == 1 || WPX == 2 || WPX == 4, "wave split");
  static_assert(PT == 32 * NB2 * WPX, "tile pixels");
  static_assert((TW == 2 || TW == 4 || TW == 8 || TW == 16) && (TH * TW) % 2 == 0, "tile shape");
  static_assert((WK - 1) * WPX * MB2 * NB2 * 16 * 64 * 4 <= MT * AROW, "partial sums fit the weight buffer");

  __shared__ __attribute__((aligned(16))) unsigned char sA[MT * AROW];
  __shared__ __attribute__((aligned(16))) unsigned char sB[NPATCH * BROW];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wpx = wv % WPX;               // pixel group of this wavefront
  const int wk = wv / WPX;                // its share of the rounds
  const int r32 = lane & 31, h = lane >> 5;

  int tile;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    tile = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  // (divisions by multiplication: a scalar division is a chain of some thirty dependent instructions, and
  // five of them in front of the first load are a tenth of a short layer's tile)
  const int tiles_s = a.tiles_n * a.tiles_y * a.tiles_x;
  const int q_s = (int)fast_div((unsigned)tile, a.magic_s), q_m = (int)fast_div((unsigned)tile, a.magic_m);
  const int tile_m = a.m_major ? q_s : tile - q_m * a.tiles_m;
  const int rest = a.m_major ? tile - q_s * tiles_s : q_m;
  const int q_x = (int)fast_div((unsigned)rest, a.magic_x);
  const int q_y = (int)fast_div((unsigned)q_x, a.magic_y);
  const int tx0 = (rest - q_x * a.tiles_x) * TW;
  const int ty0 = (q_x - q_y * a.tiles_y) * TH;
  const int n0 = q_y * NI;
  const int o0 = tile_m * MT;

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t wr = make_rsrc(a.w, a.w_bytes);
  // bias values of the epilogue (register v of a 32 x 32 block: filter 8 * (v / 4) + 4 * h + v % 4), requested
  // ahead of the main loop: asked for in the epilogue, the last tiles of a layer would wait for them in full
  float4_t bias4[MB2][4];
#pragma unroll
  for (int i = 0; i < MB2; ++i)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) bias4[i][vq] = load_bias4(a.bias, a.O, o0 + i * 32 + 8 * vq + 4 * h);

  // ---- staging items (as conv_patch_kernel) ----
  unsigned b_off[NIB];
  int b_lds[NIB], b_q[NIB];
#pragma unroll
  for (int j = 0; j < NIB; ++j) {
    const int idx = t + NT * j;
    const int q = idx % NQ, pp = idx / NQ;
    const bool item = pp < NPATCH;
    const int img = pp / (PH * PW), pr = pp - img * (PH * PW);
    const int py = pr / PW, px = pr - py * PW;
    const int iy = ty0 + py - 1, ix = tx0 + px - 1, n = n0 + img;
    const bool inside = item && n < a.N && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
    b_off[j] = inside ? (unsigned)(((n * a.H + iy) * a.W + ix) * a.Cp + q * EPI) * ES : kOutOfRange;
    b_lds[j] = item ? pp * BROW + q * 16 : -1;
    b_q[j] = q;
  }
  unsigned a_off[NIA];
  int a_lds[NIA], a_q[NIA];
#pragma unroll
  for (int j = 0; j < NIA; ++j) {
    const int idx = t + NT * j;
    const int q = idx % NQ;
    const int tap = (idx / NQ) % 9;
    const int m = (idx / NQ) / 9;
    const bool item = m < MT;
    const int o = o0 + m;
    a_off[j] = (item && o < a.O) ? (unsigned)((o * 9 + tap) * a.Cp + q * EPI) * ES : kOutOfRange;
    a_lds[j] = item ? m * AROW + tap * (64 * KQ) + q * 16 : -1;
    a_q[j] = q;
  }
  uint4 breg[NIB], areg[NIA];
  auto gload = [&](int c0) {
    const unsigned soff = (unsigned)(c0 * ES);
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      const unsigned inval = (unsigned)(c0 + a_q[j] * EPI >= a.Cp) << 31;
      areg[j] = load_b128(wr, a_off[j] | inval, soff);
    }
#pragma unroll
    for (int j = 0; j < NIB; ++j) {
      const unsigned inval = (unsigned)(c0 + b_q[j] * EPI >= a.Cp) << 31;
      breg[j] = load_b128(xr, b_off[j] | inval, soff);
    }
  };
  auto lds_store = [&]() {
#pragma unroll
    for (int j = 0; j < NIA; ++j)
      if (a_lds[j] >= 0) *(uint4*)&sA[a_lds[j]] = areg[j];
#pragma unroll
    for (int j = 0; j < NIB; ++j)
      if (b_lds[j] >= 0) *(uint4*)&sB[b_lds[j]] = breg[j];
  };

  // ---- fragment addresses ----
  int b_frag[NB2];
#pragma unroll
  for (int j = 0; j < NB2; ++j) {
    const int id = wpx * (NB2 * 32) + j * 32 + r32;
    const int img = id / (TH * TW), ir = id % (TH * TW);
    const int ty = ir / TW, tx = ir % TW;
    b_frag[j] = ((img * PH + ty) * PW + tx) * BROW + h * 32;
  }
  const int a_frag = r32 * AROW + h * 32;

  float16_t acc[MB2][NB2];
#pragma unroll
  for (int i = 0; i < MB2; ++i)
#pragma unroll
    for (int j = 0; j < NB2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  int mb_count = (a.O - o0 + 31) / 32;
  mb_count = mb_count > MB2 ? MB2 : mb_count;

  // rounds [r_lo, r_hi) of every chunk are this wavefront's
  const int r_lo = wk * NR / WK, r_hi = (wk + 1) * NR / WK;

  const int nchunk = (a.Cp + CC - 1) / CC;
  auto main_loop = [&](auto mbc_tag) {
    constexpr int MBC = decltype(mbc_tag)::value;
    gload(0);
    for (int c = 0; c < nchunk; ++c) {
      __syncthreads();
      lds_store();
      __syncthreads();
      if (c + 1 < nchunk) gload((c + 1) * CC);
      uint4 af[2][MB2][2], bf[2][NB2][2];
      auto fetch = [&](int rnd, uint4 (&fa)[MB2][2], uint4 (&fb)[NB2][2]) {
        const int tap = rnd / KQ, q4 = rnd - tap * KQ;
        const int ty = tap / 3, tx = tap - ty * 3;
        const int boff = (ty * PW + tx) * BROW + q4 * 64;
        const int aoff = tap * (64 * KQ) + q4 * 64;
#pragma unroll
        for (int j = 0; j < NB2; ++j) {
          fb[j][0] = *(const uint4*)&sB[b_frag[j] + boff];
          fb[j][1] = *(const uint4*)&sB[b_frag[j] + boff + 16];
        }
#pragma unroll
        for (int i = 0; i < MBC; ++i) {
          fa[i][0] = *(const uint4*)&sA[a_frag + i * 32 * AROW + aoff];
          fa[i][1] = *(const uint4*)&sA[a_frag + i * 32 * AROW + aoff + 16];
        }
      };
      auto mma = [&](const uint4 (&fa)[MB2][2], const uint4 (&fb)[NB2][2]) {
        if constexpr (sizeof(T) == 4) {
#pragma unroll
          for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int i = 0; i < MBC; ++i) {
              const uint4& qa = fa[i][e >> 2];
              const uint32_t av = (e & 3) == 0 ? qa.x : (e & 3) == 1 ? qa.y : (e & 3) == 2 ? qa.z : qa.w;
#pragma unroll
              for (int j = 0; j < NB2; ++j) {
                const uint4& qb = fb[j][e >> 2];
                const uint32_t bv = (e & 3) == 0 ? qb.x : (e & 3) == 1 ? qb.y : (e & 3) == 2 ? qb.z : qb.w;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av), __uint_as_float(bv), acc[i][j], 0, 0, 0);
              }
            }
        } else {
#pragma unroll
          for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int i = 0; i < MBC; ++i)
#pragma unroll
              for (int j = 0; j < NB2; ++j) {
                if constexpr (std::is_same<T, _Float16>::value)
                  acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, fa[i][m]),
                                                                     __builtin_bit_cast(half8_t, fb[j][m]), acc[i][j], 0, 0, 0);
                else
                  acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[i][m]),
                                                                      __builtin_bit_cast(bf16x8_t, fb[j][m]), acc[i][j], 0, 0, 0);
              }
        }
      };
      // the operands of the next round are fetched from LDS while this one is multiplied
      if (r_lo < r_hi) fetch(r_lo, af[0], bf[0]);
      int cur = 0;
      for (int rnd = r_lo; rnd < r_hi; ++rnd) {
        if (rnd + 1 < r_hi) {
          if (cur == 0) fetch(rnd + 1, af[1], bf[1]); else fetch(rnd + 1, af[0], bf[0]);
        }
        if (cur == 0) mma(af[0], bf[0]); else mma(af[1], bf[1]);
        cur ^= 1;
      }
    }
  };
  switch (mb_count) {
    case 1: main_loop(std::integral_constant<int, 1>{}); break;
    case 2: if constexpr (MB2 >= 2) main_loop(std::integral_constant<int, 2>{}); break;
    case 3: if constexpr (MB2 >= 3) main_loop(std::integral_constant<int, 3>{}); break;
    case 4: if constexpr (MB2 >= 4) main_loop(std::integral_constant<int, 4>{}); break;
    default: break;
  }

  if constexpr (WK > 1) {
    // partial sums of the wavefronts that shared a block column meet in LDS (the staging
    // buffers are free now); the first of them adds, in a fixed order, and stores
    __syncthreads();
    float* xch = (float*)sA;
    auto slot = [&](int k, int i, int j, int v) { return ((((k - 1) * WPX + wpx) * MB2 + i) * NB2 + j) * 16 * 64 + v * 64 + lane; };
    if (wk > 0) {
#pragma unroll
      for (int i = 0; i < MB2; ++i)
#pragma unroll
        for (int j = 0; j < NB2; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) xch[slot(wk, i, j, v)] = acc[i][j][v];
    }
    __syncthreads();
    if (wk > 0) return;
#pragma unroll
    for (int k = 1; k < WK; ++k)
#pragma unroll
      for (int i = 0; i < MB2; ++i)
#pragma unroll
        for (int j = 0; j < NB2; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][j][v] += xch[slot(k, i, j, v)];
  }

  // ---- epilogue ----
  ConvArgs e;
  e.bias = a.bias; e.res = a.res; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act; e.vec_out = a.vec_out; e.pool4 = 0;
  if (!a.pool) {
#pragma unroll
    for (int j = 0; j < NB2; ++j) {
      const int id = wpx * (NB2 * 32) + j * 32 + r32;
      const int img = id / (TH * TW), ir = id % (TH * TW);
      const int oy = ty0 + ir / TW, ox = tx0 + ir % TW, n = n0 + img;
      if (n >= a.N || oy >= a.H || ox >= a.W) continue;
      const int p = (n * a.H + oy) * a.W + ox;
#pragma unroll
      for (int i = 0; i < MB2; ++i)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const float4_t four = (float4_t){acc[i][j][4 * vq], acc[i][j][4 * vq + 1], acc[i][j][4 * vq + 2], acc[i][j][4 * vq + 3]};
          nhwc_store4<T>(e, four, p, o0 + i * 32 + 8 * vq + 4 * h, bias4[i][vq]);
        }
    }
  } else {
    // bias + activation, then the max over each 2x2 window: the horizontal partner is lane
    // r32 ^ 1, the vertical one lane r32 ^ TW (a 32-pixel block holds whole row pairs of one
    // image); the even / even corner stores
    e.act = CPRUNE_ACT_NONE;
    e.bias = nullptr;
    const int hp = a.H >> 1, wp = a.W >> 1;
#pragma unroll
    for (int j = 0; j < NB2; ++j) {
      const int id = wpx * (NB2 * 32) + j * 32 + r32;
      const int img = id / (TH * TW), ir = id % (TH * TW);
      const int ty = ir / TW, tx = ir % TW;
      const int oy = ty0 + ty, ox = tx0 + tx, n = n0 + img;
      const bool writer = !((ty & 1) || (tx & 1) || n >= a.N || oy >= a.H || ox >= a.W);
      const int p = (n * hp + (oy >> 1)) * wp + (ox >> 1);
#pragma unroll
      for (int i = 0; i < MB2; ++i)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int o = o0 + i * 32 + 8 * vq + 4 * h;
          float4_t m;
          const float4_t bias = bias4[i][vq];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            float x = acc[i][j][4 * vq + c] + bias[c];
            x = apply_act(x, a.act);
            x = fmaxf(x, __shfl_xor(x, 1, 64));
            x = fmaxf(x, __shfl_xor(x, TW, 64));
            m[c] = x;
          }
          if (writer) nhwc_store4<T>(e, m, p, o, (float4_t){0.f, 0.f, 0.f, 0.f});
        }
    }
  }
}

// 32x32-block patch variants: id, mb2, nb2, wpx (wavefronts along pixels; 4 / wpx share a
// block column and split the rounds), th, tw, ni, kq
#define CPRUNE_PATCH32_LIST(X)   \
  X(0, 1, 1, 4, 8, 16, 1, 1)     \
  X(1, 2, 1, 4, 8, 16, 1, 1)     \
  X(2, 1, 1, 4, 8, 16, 1, 2)     \
  X(3, 1, 2, 4, 16, 16, 1, 1)    \
  X(4, 2, 2, 4, 16, 16, 1, 1)    \
  X(5, 1, 1, 2, 8, 8, 1, 1)      \
  X(6, 1, 1, 2, 8, 8, 1, 2)      \
  X(7, 2, 1, 2, 8, 8, 1, 1)      \
  X(8, 1, 1, 2, 4, 4, 4, 2)      \
  X(9, 1, 1, 1, 4, 8, 1, 2)      \
  X(10, 1, 1, 1, 4, 4, 2, 2)     \
  X(11, 1, 1, 1, 4, 4, 2, 1)     \
  X(12, 2, 1, 1, 4, 4, 2, 1)     \
  X(13, 1, 1, 4, 8, 8, 2, 2)

constexpr int kNumPatch32 = 14;

template <typename T>
inline void launch_patch32(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
#define CPRUNE_PATCH32_CASE(ID, MB2_, NB2_, WPX_, TH_, TW_, NI_, KQ_)                                               \
  case ID:                                                                                                          \
    hipLaunchKernelGGL((conv_patch32_kernel<T, MB2_, NB2_, WPX_, TH_, TW_, NI_, KQ_>), grid, dim3(256), 0, s, a);   \
    break;
  switch (id) { CPRUNE_PATCH32_LIST(CPRUNE_PATCH32_CASE) }
#undef CPRUNE_PATCH32_CASE
}

void launch_conv_patch32_f32(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
void launch_conv_patch32_f16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
void launch_conv_patch32_bf16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);

}  // namespace cprune
