// 3x3 / stride 1 / pad 1 convolution, channels-last, with the input staged as a
// spatial patch: the shape almost every layer of the evaluated networks has
// (all of VGG-16, the 3x3 layers of ResNet-18, the channel-sweep layer).
//
// In the implicit-GEMM kernel the B tile is an im2col tile, so every input
// element crosses L2 -> LDS nine times (once per tap).  Here a work-group owns a
// TH x TW block of output pixels of one image and MT filters; per chunk of 16
// bytes x 4 of channels it stages the (TH+2) x (TW+2) input patch ONCE, plus the
// [MT][9 taps][chunk] slice of the weights, and the nine taps are nine shifted
// views of the same patch: the B operand of tap (u, v) for output pixel (y, x)
// is the 16-byte quad at patch pixel (y + u, x + v), a compile-time offset from
// the lane's own pixel.  Staged bytes per MFMA drop ~3x against 64x64 im2col
// tiles, which is what small pruned filter counts need (few filters = little
// reuse of each staged input element).
//
// Same MFMA blocks and k-permutation as conv_nhwc_kernel (lane group g4 holds
// channels 4*g4..4*g4+3 of the chunk for both operands).  4 wavefronts split the
// pixels; each owns MB x NB accumulator blocks (NB blocks of 16 pixels = rows of
// the tile when TW = 16, row pairs when TW = 8).  One LDS buffer: while a chunk
// is multiplied, the next one is already in flight into registers.
#pragma once
#include "conv_nhwc_kernel.hpp"

namespace cprune {

struct PatchArgs {
  const void* x;
  const void* w;
  const float* bias;
  const void* res;
  void* y;
  int N, H, W, O, Cp, Cop;
  int tiles_n, tiles_y, tiles_x, tiles_m;
  unsigned x_bytes, w_bytes;
  int act, vec_out;
  int pool;   // 1: 2x2 / stride 2 max-pool fused behind the activation; y is [n][h/2][w/2][cop]
  // ceil(2^32 / d) for the divisions of the tile decode (0 when d == 1): by tiles_n * tiles_y * tiles_x, tiles_m,
  // tiles_x, tiles_y; for the independent-wavefront kernel magic_s divides by tiles_n and magic_xy by
  // tiles_x * tiles_y.  Exact while (number of groups) x (divisor) < 2^32, which the host checks.
  unsigned magic_s, magic_m, magic_x, magic_y, magic_xy;
  int m_major;  // tile order: 0 = filter tiles fastest (each chip quarter's L2 sees few input patches, all
                // weights), 1 = pixel tiles fastest (few filters, all patches): whichever operand is larger
                // is the one split between the L2s
  int Ho = 0, Wo = 0;   // stride-2 form only: the output map (H, W are the input map); tiles count blocks of it
};

// One 64-byte round of MFMAs on NS accumulator sets.  A tile with fewer than four
// accumulator blocks per wave would issue back-to-back MFMAs into the same block, each
// waiting for the one before; spreading consecutive instructions over NS sets (summed at
// the end) keeps them independent.
template <typename T, int MBC, int NB, int MB, int NS>
__device__ __forceinline__ void mma_round(const uint4 (&af)[MB], const uint4 (&bf)[NB],
                                          float4_t (&acc)[NS][MB][NB], int round) {
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int set = NS == 1 ? 0 : (NS >= 4 ? e : ((round * 4 + e) % NS));
#pragma unroll
      for (int i = 0; i < MBC; ++i) {
        const uint32_t av = e == 0 ? af[i].x : e == 1 ? af[i].y : e == 2 ? af[i].z : af[i].w;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const uint32_t bv = e == 0 ? bf[j].x : e == 1 ? bf[j].y : e == 2 ? bf[j].z : bf[j].w;
          acc[set][i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(av), __uint_as_float(bv), acc[set][i][j], 0, 0, 0);
        }
      }
    }
  } else {
    const int set = round % NS;
#pragma unroll
    for (int i = 0; i < MBC; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        if constexpr (std::is_same<T, _Float16>::value)
          acc[set][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, af[i]),
                                                                  __builtin_bit_cast(half8_t, bf[j]), acc[set][i][j], 0, 0, 0);
        else
          acc[set][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, af[i]),
                                                                   __builtin_bit_cast(bf16x8_t, bf[j]), acc[set][i][j], 0, 0, 0);
      }
  }
}

// Epilogue of the patch tilings: wavefront `wave` holds NB 16-pixel blocks (pixel id = wave * NB * 16 + j * 16 + r in
// the (image, row, column) order of a TH x TW tile) x MB filter blocks; bias, residual, activation, 16-byte
// channels-last stores, or the 2x2 / stride-2 max-pool fused behind the activation.
// bias4[i]: the four bias values of filter block i for this lane (load_bias4 at o0 + i * 16 + 4 * g4), fetched by
// the caller before its main loop: asked for here, the last tiles of a layer would wait for them in full.
template <typename T, int MB, int TH, int TW, int NB>
__device__ __forceinline__ void patch_epilogue(const PatchArgs& a, float4_t (&acc)[MB][NB], int wave, int r, int g4,
                                               int n0, int ty0, int tx0, int o0, const float4_t (&bias4)[MB]) {
  ConvArgs e;
  e.bias = a.bias; e.res = a.res; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act; e.vec_out = a.vec_out; e.pool4 = 0;
  if (!a.pool) {
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int id = wave * (NB * 16) + j * 16 + r;
      const int img = id / (TH * TW), ir = id % (TH * TW);
      const int oy = ty0 + ir / TW, ox = tx0 + ir % TW, n = n0 + img;
      if (n >= a.N || oy >= a.H || ox >= a.W) continue;
      const int p = (n * a.H + oy) * a.W + ox;
#pragma unroll
      for (int i = 0; i < MB; ++i) nhwc_store4<T>(e, acc[i][j], p, o0 + i * 16 + 4 * g4, bias4[i]);
    }
  } else {
    // bias + activation, then the max over each 2x2 window.  Horizontal partner: lane
    // r ^ 1.  Vertical partner: lane r ^ TW when a 16-pixel block holds several rows,
    // else the same lane of the neighbouring block.  The activation is monotone, so
    // max(act(.)) equals act-then-pool.  The even/even corner of each window stores.
    e.act = CPRUNE_ACT_NONE;
    e.bias = nullptr;
    const int hp = a.H >> 1, wp = a.W >> 1;
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int o = o0 + i * 16 + 4 * g4;
      float4_t v[NB];
      const float4_t bias = bias4[i];
#pragma unroll
      for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          float x = acc[i][j][c] + bias[c];
          x = apply_act(x, a.act);
          x = fmaxf(x, __shfl_xor(x, 1, 64));
          if constexpr (TW < 16) x = fmaxf(x, __shfl_xor(x, TW, 64));
          v[j][c] = x;
        }
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        float4_t m = v[j];
        if constexpr (TW == 16) {
#pragma unroll
          for (int c = 0; c < 4; ++c) m[c] = fmaxf(m[c], v[j ^ 1][c]);
        }
        const int id = wave * (NB * 16) + j * 16 + r;
        const int img = id / (TH * TW), ir = id % (TH * TW);
        const int ty = ir / TW, tx = ir % TW;
        const int oy = ty0 + ty, ox = tx0 + tx, n = n0 + img;
        if ((ty & 1) || (tx & 1) || n >= a.N || oy >= a.H || ox >= a.W) continue;
        const int p = (n * hp + (oy >> 1)) * wp + (ox >> 1);
        nhwc_store4<T>(e, m, p, o, (float4_t){0.f, 0.f, 0.f, 0.f});
      }
    }
  }
}

template <typename T, int MB>
__device__ __forceinline__ void load_tile_bias(const PatchArgs& a, int o0, int g4, float4_t (&bias4)[MB]) {
#pragma unroll
  for (int i = 0; i < MB; ++i) bias4[i] = load_bias4(a.bias, a.O, o0 + i * 16 + 4 * g4);
}

 // S: stride of the window (1, or 2 for the layers that halve the map: the patch is then (TH - 1) * 2 + 3 rows
// by (TW - 1) * 2 + 3 columns and a lane's tap is the same compile-time offset from twice its pixel position)
template <typename T, int MB, int TH, int TW, int NI, int KQ, int KS, int S>
__device__ __forceinline__ void patch_body(const PatchArgs& a) {
  constexpr int NT = 256 * KS;            // KS groups of 4 wavefronts share a tile: each takes 1/KS of the rounds
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;            // elements per quad
  constexpr int CC = 4 * EPI * KQ;        // channels per chunk (KQ rounds of 64 bytes)
  constexpr int NQ = 4 * KQ;              // quads per pixel per chunk
  constexpr int PT = TH * TW * NI;        // output pixels per tile (NI images x TH x TW)
  constexpr int NB = PT / 64;             // 16-pixel blocks per wave
  constexpr int MT = MB * 16;
  constexpr int PW = (TW - 1) * S + 3, PH = (TH - 1) * S + 3;
  constexpr int NPATCH = NI * PH * PW;
  constexpr int BROW = 64 * KQ + 16;      // patch pixel: the chunk's channels + 16 pad
  constexpr int AROW = 9 * 64 * KQ + 16;  // filter row: 9 taps x chunk + 16 pad
  constexpr int NIB = (NPATCH * NQ + NT - 1) / NT;
  constexpr int NIA = (MT * 9 * NQ + NT - 1) / NT;
  constexpr int NS = (MB * (PT / 64) >= 4) ? 1 : 4 / (MB * (PT / 64));  // accumulator sets
  static_assert(PT % 64 == 0 && (TW == 2 || TW == 4 || TW == 8 || TW == 16) && (16 % TW == 0), "tile shape");
  static_assert(S == 1 || (S == 2 && NI == 1 && KS == 1), "stride");

  __shared__ __attribute__((aligned(16))) unsigned char sA[MT * AROW];
  __shared__ __attribute__((aligned(16))) unsigned char sB[NPATCH * BROW];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = (t >> 6) & 3;          // pixel group of this wavefront
  const int kgrp = t >> 8;                // which share of the rounds it multiplies
  const int r = lane & 15, g4 = lane >> 4;

  // tile decode; each XCD (own L2) gets one contiguous stretch of the tile order
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
  float4_t bias4[MB];
  load_tile_bias<T, MB>(a, o0, g4, bias4);

  // ---- staging items ----
  unsigned b_off[NIB];   // byte offset of (patch pixel, quad) at chunk 0, kOutOfRange outside the image
  int b_lds[NIB], b_q[NIB];
#pragma unroll
  for (int j = 0; j < NIB; ++j) {
    const int idx = t + NT * j;
    const int q = idx % NQ, pp = idx / NQ;
    const bool item = pp < NPATCH;
    const int img = pp / (PH * PW), pr = pp - img * (PH * PW);
    const int py = pr / PW, px = pr - py * PW;
    const int iy = ty0 * S + py - 1, ix = tx0 * S + px - 1, n = n0 + img;
    const bool inside = item && n < a.N && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
    b_off[j] = inside ? (unsigned)(((n * a.H + iy) * a.W + ix) * a.Cp + q * EPI) * ES : kOutOfRange;
    b_lds[j] = item ? pp * BROW + q * 16 : NPATCH * BROW - 16;   // no item: the last row's pad, which nobody reads
    b_q[j] = q;
  }
  unsigned a_off[NIA];   // byte offset of (filter, tap, quad) at chunk 0
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
    a_lds[j] = item ? m * AROW + tap * (64 * KQ) + q * 16 : MT * AROW - 16;
    a_q[j] = q;
  }

  uint4 breg[NIB], areg[NIA];
  auto gload = [&](int c0) {   // c0: first channel of the chunk
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
    for (int j = 0; j < NIA; ++j) *(uint4*)&sA[a_lds[j]] = areg[j];   // unconditional: a branch per item costs more
#pragma unroll
    for (int j = 0; j < NIB; ++j) *(uint4*)&sB[b_lds[j]] = breg[j];
  };

  // ---- fragment addresses: lane's pixel inside the patch (tap (0,0) corner) ----
  int b_frag[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int id = wave * (NB * 16) + j * 16 + r;
    const int img = id / (TH * TW), ir = id % (TH * TW);
    const int ty = ir / TW, tx = ir % TW;
    b_frag[j] = ((img * PH + ty * S) * PW + tx * S) * BROW + g4 * 16;
  }
  const int a_frag = r * AROW + g4 * 16;

  float4_t accs[NS][MB][NB];
#pragma unroll
  for (int q = 0; q < NS; ++q)
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) accs[q][i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};

  int mb_count = (a.O - o0 + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;

  const int nchunk = (a.Cp + CC - 1) / CC;
  auto main_loop = [&](auto mbc_tag) {
    constexpr int MBC = decltype(mbc_tag)::value;
    gload(0);
    for (int c = 0; c < nchunk; ++c) {
      __syncthreads();            // everyone is done reading the previous chunk
      lds_store();
      __syncthreads();
      if (c + 1 < nchunk) gload((c + 1) * CC);
      // the operands of round r + 1 are fetched from LDS while round r is multiplied;
      // wave group kgrp takes rounds [kgrp * NR / KS, (kgrp + 1) * NR / KS)
      constexpr int NR = 9 * KQ;
      // ST = 1: every round of [LO, HI).  ST = KQ: only the first 64-byte round of each tap, for a
      // last chunk whose channels end inside that round (the rest of the chunk is zero fill)
      auto rounds = [&](auto lo_tag, auto hi_tag, auto step_tag) {
        constexpr int LO = decltype(lo_tag)::value, HI = decltype(hi_tag)::value, ST = decltype(step_tag)::value;
        // fragments are fetched PF rounds ahead of their use (PF + 1 register sets)
        constexpr int PF = 1;
        uint4 af[PF + 1][MB], bf[PF + 1][NB];
        auto fetch = [&](int rnd, uint4 (&fa)[MB], uint4 (&fb)[NB]) {
          const int tap = rnd / KQ, q4 = rnd % KQ;
          const int boff = ((tap / 3) * PW + (tap % 3)) * BROW + q4 * 64;
#pragma unroll
          for (int j = 0; j < NB; ++j) fb[j] = *(const uint4*)&sB[b_frag[j] + boff];
#pragma unroll
          for (int i = 0; i < MBC; ++i) fa[i] = *(const uint4*)&sA[a_frag + i * 16 * AROW + tap * (64 * KQ) + q4 * 64];
        };
#pragma unroll
        for (int p = 0; p < PF; ++p)
          if (LO + p * ST < HI) fetch(LO + p * ST, af[p], bf[p]);
#pragma unroll
        for (int rnd = LO; rnd < HI; rnd += ST) {
          const int idx = (rnd - LO) / ST;
          if (rnd + PF * ST < HI) fetch(rnd + PF * ST, af[(idx + PF) % (PF + 1)], bf[(idx + PF) % (PF + 1)]);
          // Multi-image tiles serve small maps, whose grids leave one wavefront per SIMD: there
          // the fetch is pinned ahead of the multiplies (left alone, the scheduler sinks every LDS
          // read to just before its first use and the four wavefronts take turns on the LDS and
          // the matrix pipes).  With many resident wavefronts the scheduler's own order is faster.
          if constexpr (NI > 1) __builtin_amdgcn_sched_barrier(0);
          // a wavefront that has its operands goes first: with several tiles resident, their staging instructions
          // otherwise take issue slots between the MFMAs (1-3 % on the layers of this kernel)
          __builtin_amdgcn_s_setprio(1);
          mma_round<T, MBC, NB, MB, NS>(af[idx % (PF + 1)], bf[idx % (PF + 1)], accs, idx);
          __builtin_amdgcn_s_setprio(0);
          if constexpr (NI > 1) __builtin_amdgcn_sched_barrier(0);
        }
      };
      using One = std::integral_constant<int, 1>;
      if constexpr (KS == 1) {
        if (KQ > 1 && c + 1 == nchunk && (a.Cp - c * CC) * ES <= 64)
          rounds(std::integral_constant<int, 0>{}, std::integral_constant<int, NR>{}, std::integral_constant<int, KQ>{});
        else
          rounds(std::integral_constant<int, 0>{}, std::integral_constant<int, NR>{}, One{});
      } else {
        constexpr int MID = (NR + 1) / 2;
        if (kgrp == 0) rounds(std::integral_constant<int, 0>{}, std::integral_constant<int, MID>{}, One{});
        else rounds(std::integral_constant<int, MID>{}, std::integral_constant<int, NR>{}, One{});
      }
    }
  };
  switch (mb_count) {
#define CPRUNE_MBC_CASE(V) \
  case V: if constexpr (MB >= V) main_loop(std::integral_constant<int, V>{}); break;
    CPRUNE_MBC_CASE(1) CPRUNE_MBC_CASE(2) CPRUNE_MBC_CASE(3) CPRUNE_MBC_CASE(4)
    CPRUNE_MBC_CASE(5) CPRUNE_MBC_CASE(6) CPRUNE_MBC_CASE(7) CPRUNE_MBC_CASE(8)
#undef CPRUNE_MBC_CASE
    default: break;
  }

  float4_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      acc[i][j] = accs[0][i][j];
#pragma unroll
      for (int q = 1; q < NS; ++q) acc[i][j] += accs[q][i][j];
    }

  if constexpr (KS > 1) {
    // the second wave group hands its sums over through LDS (the staging buffers are free now)
    __syncthreads();
    float4_t* xch = (float4_t*)sA + (size_t)wave * (MB * NB * 64) + lane;
    static_assert(4 * MB * NB * 64 * 16 <= MT * AROW, "exchange fits the weight buffer");
    if (kgrp == 1) {
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) xch[(i * NB + j) * 64] = acc[i][j];
    }
    __syncthreads();
    if (kgrp == 1) return;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] += xch[(i * NB + j) * 64];
  }

  // ---- epilogue ----
  if constexpr (S == 1) {
    patch_epilogue<T, MB, TH, TW, NB>(a, acc, wave, r, g4, n0, ty0, tx0, o0, bias4);
  } else {
    PatchArgs out = a;          // the epilogue indexes the map it writes
    out.H = a.Ho; out.W = a.Wo;
    patch_epilogue<T, MB, TH, TW, NB>(out, acc, wave, r, g4, n0, ty0, tx0, o0, bias4);
  }
}

template <typename T, int MB, int TH, int TW, int NI, int KQ, int KS>
__global__ __launch_bounds__(256 * KS) void conv_patch_kernel(PatchArgs a) {
  patch_body<T, MB, TH, TW, NI, KQ, KS, 1>(a);
}

// 3x3 / stride 2 / pad 1 (the layers that halve the map between the stages of a residual network): the same
// kernel on a patch of twice the extent.  An input element is still staged once per tile instead of once per tap
// that touches it, as the im2col tiles of the general kernel do.
template <typename T, int MB, int TH, int TW, int KQ>
__global__ __launch_bounds__(256) void conv_patch_s2_kernel(PatchArgs a) {
  patch_body<T, MB, TH, TW, 1, KQ, 1, 2>(a);
}

// Patch variants: id, mb, th, tw, ni (images per tile, for maps smaller than the tile; two images of a 7x7 map
// share an 8x8 x 2 tile),
// kq (64-byte channel rounds per chunk), ks (wave groups per tile: 2 = eight wavefronts,
// each group multiplying half of every chunk's rounds; for layers with about as many
// tiles as compute units, where one group per unit leaves the MFMA pipe waiting)
#define CPRUNE_PATCH_LIST(X) \
  X(0, 1, 8, 8, 1, 1, 1)    \
  X(1, 2, 8, 8, 1, 1, 1)    \
  X(2, 4, 8, 8, 1, 1, 1)    \
  X(3, 2, 8, 16, 1, 1, 1)   \
  X(4, 4, 8, 16, 1, 1, 1)   \
  X(5, 2, 16, 16, 1, 1, 1)  \
  X(6, 4, 16, 16, 1, 1, 1)  \
  X(7, 1, 16, 16, 1, 1, 1)  \
  X(8, 1, 4, 4, 4, 1, 1)    \
  X(9, 2, 4, 4, 4, 2, 1)    \
  X(10, 1, 2, 2, 16, 1, 1)  \
  X(11, 2, 2, 2, 16, 1, 1)  \
  X(12, 1, 8, 8, 1, 2, 1)   \
  X(13, 2, 8, 8, 1, 2, 1)   \
  X(14, 1, 4, 4, 4, 2, 1)   \
  X(15, 1, 2, 2, 16, 2, 1)  \
  X(16, 1, 8, 8, 1, 2, 2)   \
  X(17, 1, 4, 4, 4, 2, 2)   \
  X(18, 2, 8, 8, 1, 2, 2)   \
  X(19, 2, 4, 4, 4, 2, 2)   \
  X(20, 1, 2, 2, 16, 2, 2)  \
  X(21, 4, 8, 8, 1, 1, 2)   \
  X(22, 2, 8, 16, 1, 1, 2)  \
  X(23, 2, 8, 8, 2, 2, 1)

constexpr int kNumPatch = 24;

template <typename T>
inline void launch_patch(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
#define CPRUNE_PATCH_CASE(ID, MB_, TH_, TW_, NI_, KQ_, KS_)                                                      \
  case ID:                                                                                                       \
    hipLaunchKernelGGL((conv_patch_kernel<T, MB_, TH_, TW_, NI_, KQ_, KS_>), grid, dim3(256 * KS_), 0, s, a);    \
    break;
  switch (id) { CPRUNE_PATCH_LIST(CPRUNE_PATCH_CASE) }
#undef CPRUNE_PATCH_CASE
}

// Stride-2 variants: id, mb, th, tw, kq
#define CPRUNE_PATCH_S2_LIST(X) \
  X(0, 1, 8, 8, 1)   \
  X(1, 2, 8, 8, 1)   \
  X(2, 4, 8, 8, 1)   \
  X(3, 2, 8, 16, 1)  \
  X(4, 4, 8, 16, 1)  \
  X(5, 2, 8, 8, 2)   \
  X(6, 4, 8, 8, 2)

constexpr int kNumPatchS2 = 7;

template <typename T>
inline void launch_patch_s2(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
#define CPRUNE_PATCH_S2_CASE(ID, MB_, TH_, TW_, KQ_)                                              \
  case ID:                                                                                        \
    hipLaunchKernelGGL((conv_patch_s2_kernel<T, MB_, TH_, TW_, KQ_>), grid, dim3(256), 0, s, a);  \
    break;
  switch (id) { CPRUNE_PATCH_S2_LIST(CPRUNE_PATCH_S2_CASE) }
#undef CPRUNE_PATCH_S2_CASE
}

void launch_conv_patch_f32(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
void launch_conv_patch_s2_f32(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
void launch_conv_patch_s2_f16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
void launch_conv_patch_s2_bf16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
void launch_conv_patch_f16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
void launch_conv_patch_bf16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);

}  // namespace cprune
