// First layer of an ImageNet-style network in 16-bit data: 7 x 7 / stride 2 / pad 3 convolution of an
// NCHW image with at most 3 channels, channels-last output, optionally with the 3 x 3 / stride 2 / pad 1
// max-pool that follows it in the same kernel.
//
// The general first-layer kernel builds a lane's B operand element by element from a planar patch (one
// 2-byte LDS read per k).  Here the patch is staged pixel-major, four channels per pixel (the fourth is
// zero), and the reduction is ordered (window row, window column, channel) with the window row padded to 8
// columns: one MFMA round of k = 32 is then one window row, and a lane's 16-byte quad of it is two
// neighbouring pixels of the patch, 16-byte aligned because the output column stride is 2 pixels.  One LDS
// read per operand and round; 7 rounds; 147 of the 224 multiplied terms are real (the rest meet zero
// weights), which costs nothing noticeable at this data type.  A third of the LDS instructions of the general
// kernel; by itself that only draws level with it, because in 16-bit data this layer's time is the vector work
// around the MFMAs (bias, activation, conversion, addresses) and waiting.  What pays is the pool:
//
// A work-group owns a 16 x 16 block of conv outputs and MT = 16 * MB filters, keeps its weight tile in
// LDS and walks over several blocks (the next block's patch travels to registers meanwhile).  With the
// pool fused the block sits at conv offset (2 * py0 - 1, 2 * px0 - 1) and yields the 7 x 7 pooled
// outputs whose windows lie inside it (rows and columns 0..14; the sixteenth is computed and not used):
// activated conv outputs go to LDS in the activation type, as the separate layer would store them, and
// the pooled maxima are written with 16-byte stores.  The conv map, the largest tensor of such a network,
// never reaches memory, and the pool's launch goes away.
#pragma once
#include "conv_patch_kernel.hpp"

namespace cprune {

template <typename T, int MB, int POOL>
__global__ __launch_bounds__(256) void conv_stem7_kernel(StemArgs a) {
  static_assert(sizeof(T) == 2, "16-bit data");
  constexpr int NT = 256;
  constexpr int K = 7;
  constexpr int TH = 16, NB = 4;              // wave w owns conv rows 4w .. 4w + 3 of the block, 16 columns each
  constexpr int MT = MB * 16;
  constexpr int PH = (TH - 1) * 2 + K;        // 37 patch rows
  constexpr int PWC = 40;                     // patch columns (38 used), 4 channels x 2 bytes each
  constexpr int PROW = PWC * 8;               // bytes per patch row
  constexpr int KP = K * 32;                  // k per filter: 7 window rows x (8 columns x 4 channels)
  constexpr int AROW = KP * 2 + 16;           // bytes per weight row
  constexpr int CROW = MT * 2 + 16;           // bytes per pixel of the conv block kept for the pool
  constexpr int NL = (PH * (PWC / 2) + NT - 1) / NT;   // pixel pairs of the patch per thread

  __shared__ __attribute__((aligned(16))) unsigned char sA[MT * AROW];
  __shared__ __attribute__((aligned(16))) unsigned char sP[PH * PROW];
  __shared__ __attribute__((aligned(16))) unsigned char sC[POOL ? 256 * CROW : 16];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int r = lane & 15, g4 = lane >> 4;

  int worker;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    worker = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  const int o0 = blockIdx.y * MT;
  const unsigned short* __restrict__ xg = (const unsigned short*)a.x;

  // ---- once per worker: the weight tile (16-byte copies of packed rows) ----
  {
    constexpr int QROW = KP * 2 / 16;
    const uint4* __restrict__ wq = (const uint4*)a.w + (size_t)o0 * QROW;
    for (int idx = t; idx < MT * QROW; idx += NT) {
      const int m = idx / QROW, q = idx - m * QROW;
      *(uint4*)&sA[m * AROW + q * 16] = wq[idx];
    }
  }
  float4_t bias4[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) bias4[i] = load_bias4(a.bias, a.O, o0 + i * 16 + 4 * g4);

  int b_frag[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) b_frag[j] = (2 * (4 * wave + j)) * PROW + 16 * (r + g4);
  const int a_frag = r * AROW + g4 * 16;
  int mb_count = (a.O - o0 + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;

  // block -> (image, conv origin of the 16 x 16 block)
  auto origin = [&](int tile, int& n, int& cy0, int& cx0) {
    const int rest = (int)fast_div((unsigned)tile, a.magic_x);
    n = (int)fast_div((unsigned)rest, a.magic_y);
    const int tx = tile - rest * a.tiles_x, ty = rest - n * a.tiles_y;
    cy0 = POOL ? 14 * ty - 1 : 16 * ty;
    cx0 = POOL ? 14 * tx - 1 : 16 * tx;
  };

  // the patch of the next block travels to registers while this one is multiplied: per thread NL pairs of
  // neighbouring pixels (an even input column and the next), one 32-bit word per channel
  uint32_t pre[NL][3];
  const bool w_even = (a.W & 1) == 0;
  auto load_patch = [&](int tile) {
    int n, cy0, cx0;
    origin(tile, n, cy0, cx0);
    const int iy0 = 2 * cy0 - 3, ix0 = 2 * cx0 - 4;   // ix0 is even: a pair never straddles the image edge when W is even
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int idx = t + NT * j;
      const int pr = idx / (PWC / 2), pp = idx - pr * (PWC / 2);
      const int iy = iy0 + pr, ix = ix0 + 2 * pp;
      const bool row_ok = pr < PH && (unsigned)iy < (unsigned)a.H;
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        uint32_t v = 0;
        if (row_ok && c < a.C) {
          const size_t base = ((size_t)(n * a.C + c) * a.H + iy) * a.W;
          if (w_even) {
            if ((unsigned)ix < (unsigned)a.W) v = *(const uint32_t*)(xg + base + ix);
          } else {
            if ((unsigned)ix < (unsigned)a.W) v = xg[base + ix];
            if ((unsigned)(ix + 1) < (unsigned)a.W) v |= (uint32_t)xg[base + ix + 1] << 16;
          }
        }
        pre[j][c] = v;
      }
    }
  };
  auto store_patch = [&]() {
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int idx = t + NT * j;
      if (idx >= PH * (PWC / 2)) continue;
      uint4 q;   // pixel 0: (c0, c1, c2, 0), pixel 1 the same
      q.x = (pre[j][0] & 0xffffu) | (pre[j][1] << 16);
      q.y = pre[j][2] & 0xffffu;
      q.z = (pre[j][0] >> 16) | (pre[j][1] & 0xffff0000u);
      q.w = pre[j][2] >> 16;
      *(uint4*)&sP[idx * 16] = q;   // (pr * (PWC / 2) + pp) * 16 = pr * PROW + pp * 16
    }
  };

  ConvArgs e;
  e.bias = a.bias; e.res = nullptr; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act; e.vec_out = a.vec_out; e.pool4 = 0;

  // Order inside a block: multiply; barrier; the NEXT block's patch goes from registers to LDS; this block's
  // stores; barrier; the loads of the block after next (so the wait for a patch never has stores issued just
  // before it in front of it: loads and stores share one in-order counter).
  const int ptiles = a.N * a.tiles_y * a.tiles_x;
  if (worker < ptiles) {
    load_patch(worker);
    store_patch();
    __syncthreads();
    if (worker + (int)gridDim.x < ptiles) load_patch(worker + gridDim.x);
  }
  for (int tile = worker; tile < ptiles; tile += gridDim.x) {
    int n, cy0, cx0;
    origin(tile, n, cy0, cx0);
    const bool more = tile + (int)gridDim.x < ptiles;

    // ---- multiply: one round per window row ----
    float4_t accs[1][MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) accs[0][i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};
    auto main_loop = [&](auto mbc_tag) {
      constexpr int MBC = decltype(mbc_tag)::value;
      uint4 af[2][MB], bf[2][NB];
      auto fetch = [&](int ky, uint4 (&fa)[MB], uint4 (&fb)[NB]) {
#pragma unroll
        for (int j = 0; j < NB; ++j) fb[j] = *(const uint4*)&sP[b_frag[j] + ky * PROW];
#pragma unroll
        for (int i = 0; i < MBC; ++i) fa[i] = *(const uint4*)&sA[a_frag + i * 16 * AROW + ky * 64];
      };
      fetch(0, af[0], bf[0]);
#pragma unroll
      for (int ky = 0; ky < K; ++ky) {
        if (ky + 1 < K) fetch(ky + 1, af[(ky + 1) & 1], bf[(ky + 1) & 1]);
        mma_round<T, MBC, NB, MB, 1>(af[ky & 1], bf[ky & 1], accs, ky);
      }
    };
    switch (mb_count) {
      case 1: main_loop(std::integral_constant<int, 1>{}); break;
      case 2: if constexpr (MB >= 2) main_loop(std::integral_constant<int, 2>{}); break;
      case 3: if constexpr (MB >= 3) main_loop(std::integral_constant<int, 3>{}); break;
      case 4: if constexpr (MB >= 4) main_loop(std::integral_constant<int, 4>{}); break;
      default: break;
    }

    if constexpr (POOL) {
      // activated conv outputs in the activation type, pixel-major
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          T h[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) h[c] = Elem<T>::from_f32(apply_act(accs[0][i][j][c] + bias4[i][c], a.act));
          *(uint2*)&sC[((4 * wave + j) * 16 + r) * CROW + (i * 16 + 4 * g4) * 2] = *(const uint2*)h;
        }
    }
    __syncthreads();          // everyone is done reading the patch (and the conv block is complete)
    if (more) store_patch();

    if constexpr (!POOL) {
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int oy = cy0 + 4 * wave + j, ox = cx0 + r;
        if (oy >= a.Ho || ox >= a.Wo) continue;
        const int p = (n * a.Ho + oy) * a.Wo + ox;
#pragma unroll
        for (int i = 0; i < MB; ++i) nhwc_store4<T>(e, accs[0][i][j], p, o0 + i * 16 + 4 * g4, bias4[i]);
      }
    } else {
      // the 3 x 3 / stride 2 maxima of the conv block
      constexpr int QN = MT / 8;                  // 16-byte channel groups per pixel
      const int py0 = (cy0 + 1) >> 1, px0 = (cx0 + 1) >> 1;
      for (int idx = t; idx < 49 * QN; idx += NT) {
        const int q = idx % QN, pp = idx / QN;
        const int pyl = pp / 7, pxl = pp - pyl * 7;
        const int py = py0 + pyl, px = px0 + pxl;
        if (py >= a.Hp || px >= a.Wp || o0 + q * 8 >= a.Cop) continue;
        float m[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) m[c] = -INFINITY;
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
#pragma unroll
          for (int dx = 0; dx < 3; ++dx) {
            const int cyl = 2 * pyl + dy, cxl = 2 * pxl + dx;
            if ((unsigned)(cy0 + cyl) >= (unsigned)a.Ho || (unsigned)(cx0 + cxl) >= (unsigned)a.Wo) continue;
            const uint4 v = *(const uint4*)&sC[(cyl * 16 + cxl) * CROW + q * 16];
            const T* hv = (const T*)&v;
#pragma unroll
            for (int c = 0; c < 8; ++c) m[c] = fmaxf(m[c], Elem<T>::to_f32(hv[c]));
          }
        T h[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) h[c] = Elem<T>::from_f32(m[c]);
        *(uint4*)((T*)a.y + ((size_t)(n * a.Hp + py) * a.Wp + px) * a.Cop + o0 + q * 8) = *(const uint4*)h;
      }
    }
    __syncthreads();          // the next patch is in place; the conv block may be overwritten
    if (tile + 2 * (int)gridDim.x < ptiles) load_patch(tile + 2 * gridDim.x);
  }
}

template <typename T>
inline int launch_stem7(int mb, int pool, dim3 grid, hipStream_t s, const StemArgs& a) {
#define CPRUNE_STEM7(MB_, POOL_)                                                                   \
  if (mb == MB_ && pool == POOL_) {                                                                \
    hipLaunchKernelGGL((conv_stem7_kernel<T, MB_, POOL_>), grid, dim3(256), 0, s, a);              \
    return CPRUNE_OK;                                                                              \
  }
  CPRUNE_STEM7(2, 0) CPRUNE_STEM7(2, 1) CPRUNE_STEM7(4, 0) CPRUNE_STEM7(4, 1)
#undef CPRUNE_STEM7
  return CPRUNE_ERR_UNSUPPORTED;
}

}  // namespace cprune
