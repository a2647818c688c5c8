// First layer of a network: k x k convolution of an NCHW input with at most 3 channels
// (the image), channels-last output.  The whole reduction (c_in * k * k <= 147 terms) fits
// in LDS at once, so there is no chunk loop: a work-group stages the input patch of its
// 8 x 16 output pixels (every channel, halo included) and all the weights of its filter
// tile once, then multiplies.  The im2col tile is never materialised: a lane builds its B
// operand for a round of k from the patch through a small table of patch offsets (one per
// k, shared by all pixels), so each input element is read from global memory once per
// work-group instead of once per tap that touches it.  A work-group keeps its weight tile
// and walks over several pixel blocks (grid.x workers share the blocks round-robin), so the
// weights are staged once per worker; they arrive already padded and laid out for 16-byte
// copies ([filter tile rows][KP], prepared when the handle is built).
//
// Rows of the weight tile are k-contiguous in the weights' own (c, u, v) order; the k axis
// is padded with zero weights to a whole number of MFMA rounds.  Same 16x16 MFMA blocks,
// lane layout and k-permutation as the other dense kernels: lane group g4 takes the g4-th
// 16-byte quad of a 64-byte round for both operands.
#pragma once
#include "conv_nhwc_kernel.hpp"

namespace cprune {

template <typename T, int K, int S, int MB>
__global__ __launch_bounds__(256) void conv_stem_kernel(StemArgs a) {
  constexpr int NT = 256;
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;                 // elements per 16-byte quad
  constexpr int RK = 4 * EPI;                  // k per MFMA round (64 bytes)
  constexpr int TH = 8, TW = 16, NB = 2;       // 128 pixels: wave w owns output rows 2w, 2w + 1
  constexpr int MT = MB * 16;
  constexpr int CMAX = 3;
  constexpr int PH = (TH - 1) * S + K, PW = (TW - 1) * S + K;
  constexpr int PWP = (PW + 3) / 4 * 4;        // patch row stride (elements)
  constexpr int KMAX = CMAX * K * K;
  constexpr int KP = (KMAX + RK - 1) / RK * RK;  // k padded to whole rounds
  constexpr int NR = KP / RK;
  constexpr int AROW = KP * ES + 16;           // bytes per weight row
  static_assert(MT * AROW + CMAX * PH * PWP * ES + KP * 4 <= 65536, "LDS budget");

  __shared__ __attribute__((aligned(16))) unsigned char sA[MT * AROW];
  __shared__ __attribute__((aligned(16))) T sP[CMAX * PH * PWP];
  __shared__ __attribute__((aligned(16))) int sT[KP];

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
  const int tile_m = blockIdx.y;
  const int o0 = tile_m * MT;
  const int ktot = a.C * K * K;
  const T* __restrict__ xg = (const T*)a.x;

  // ---- once per worker: offset table and the weight tile (16-byte copies of packed rows) ----
  for (int k = t; k < KP; k += NT) {
    int off = 0;
    if (k < ktot) {
      const int c = k / (K * K), uv = k - c * (K * K);
      const int u = uv / K, v = uv - u * K;
      off = (c * PH + u) * PWP + v;
    }
    sT[k] = off;
  }
  {
    constexpr int QROW = KP * ES / 16;       // 16-byte quads per packed row
    const uint4* __restrict__ wq = (const uint4*)a.w + (size_t)o0 * QROW;
    for (int idx = t; idx < MT * QROW; idx += NT) {
      const int m = idx / QROW, q = idx - m * QROW;
      *(uint4*)&sA[m * AROW + q * 16] = wq[idx];
    }
  }

  int pbase[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) pbase[j] = ((2 * wave + j) * S) * PWP + r * S;
  const int a_frag = r * AROW + g4 * 16;
  int mb_count = (a.O - o0 + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;
  ConvArgs e;
  e.bias = a.bias; e.res = nullptr; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act; e.vec_out = a.vec_out;

  // the patch of the next pixel block travels to registers while this one is multiplied
  constexpr int NL = (CMAX * PH * PWP + NT - 1) / NT;
  T pre[NL];
  const int plimit = a.C * PH * PWP;
  auto load_patch = [&](int tile) {
    const int rest = (int)fast_div((unsigned)tile, a.magic_x);   // multiply-high: no scalar division chains
    const int n = (int)fast_div((unsigned)rest, a.magic_y);
    const int tx0 = (tile - rest * a.tiles_x) * TW;
    const int ty0 = (rest - n * a.tiles_y) * TH;
    const int iy0 = ty0 * S - a.pad, ix0 = tx0 * S - a.pad;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int idx = t + NT * j;
      const int px = idx % PWP;
      const int cy = idx / PWP;
      const int py = cy % PH, c = cy / PH;
      const int iy = iy0 + py, ix = ix0 + px;
      T val = (T)0.0f;
      if (idx < plimit && px < PW && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W)
        val = xg[((size_t)(n * a.C + c) * a.H + iy) * a.W + ix];
      pre[j] = val;
    }
  };

  const int ptiles = a.N * a.tiles_y * a.tiles_x;
  if (worker < ptiles) load_patch(worker);
  for (int tile = worker; tile < ptiles; tile += gridDim.x) {
    const int rest = (int)fast_div((unsigned)tile, a.magic_x);   // multiply-high: no scalar division chains
    const int n = (int)fast_div((unsigned)rest, a.magic_y);
    const int tx0 = (tile - rest * a.tiles_x) * TW;
    const int ty0 = (rest - n * a.tiles_y) * TH;

    __syncthreads();          // the previous block's reads of the patch are done
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const int idx = t + NT * j;
      if (idx < CMAX * PH * PWP) sP[idx] = pre[j];
    }
    __syncthreads();
    if (tile + (int)gridDim.x < ptiles) load_patch(tile + gridDim.x);

    // ---- multiply ----
    float4_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};
    auto main_loop = [&](auto mbc_tag) {
      constexpr int MBC = decltype(mbc_tag)::value;
#pragma unroll
      for (int rnd = 0; rnd < NR; ++rnd) {
        int offs[EPI];
#pragma unroll
        for (int q = 0; q < EPI / 4; ++q) {
          const int4 o4 = *(const int4*)&sT[rnd * RK + g4 * EPI + 4 * q];
          offs[4 * q] = o4.x; offs[4 * q + 1] = o4.y; offs[4 * q + 2] = o4.z; offs[4 * q + 3] = o4.w;
        }
        uint4 af[MB], bf[NB];
#pragma unroll
        for (int i = 0; i < MBC; ++i) af[i] = *(const uint4*)&sA[a_frag + i * 16 * AROW + rnd * 64];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          T* be = reinterpret_cast<T*>(&bf[j]);
#pragma unroll
          for (int e2 = 0; e2 < EPI; ++e2) be[e2] = sP[pbase[j] + offs[e2]];
        }
        mma_slab<T, MBC, NB, MB>(af, bf, acc);
      }
    };
    switch (mb_count) {
      case 1: main_loop(std::integral_constant<int, 1>{}); break;
      case 2: if constexpr (MB >= 2) main_loop(std::integral_constant<int, 2>{}); break;
      case 3: if constexpr (MB >= 3) main_loop(std::integral_constant<int, 3>{}); break;
      case 4: if constexpr (MB >= 4) main_loop(std::integral_constant<int, 4>{}); break;
      default: break;
    }

    // ---- epilogue: bias, activation, channels-last store ----
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int oy = ty0 + 2 * wave + j, ox = tx0 + r;
      if (oy >= a.Ho || ox >= a.Wo) continue;
      const int p = (n * a.Ho + oy) * a.Wo + ox;
#pragma unroll
      for (int i = 0; i < MB; ++i) nhwc_store4<T>(e, acc[i][j], p, o0 + i * 16 + 4 * g4);
    }
  }
}

// Instantiations: (k, stride) in {(3, 1), (3, 2), (7, 2)}, MB in {2, 4}
template <typename T>
inline int launch_stem(int k, int stride, int mb, dim3 grid, hipStream_t s, const StemArgs& a) {
#define CPRUNE_STEM(K_, S_, MB_)                                                                  \
  if (k == K_ && stride == S_ && mb == MB_) {                                                     \
    hipLaunchKernelGGL((conv_stem_kernel<T, K_, S_, MB_>), grid, dim3(256), 0, s, a);             \
    return CPRUNE_OK;                                                                             \
  }
  CPRUNE_STEM(3, 1, 2) CPRUNE_STEM(3, 1, 4) CPRUNE_STEM(3, 2, 2) CPRUNE_STEM(3, 2, 4)
  CPRUNE_STEM(7, 2, 2) CPRUNE_STEM(7, 2, 4)
#undef CPRUNE_STEM
  return CPRUNE_ERR_UNSUPPORTED;
}

}  // namespace cprune
