// Depthwise k x k convolution (+ bias + activation) fused with the 1x1 convolution that
// consumes it: the second half of an inverted-residual block (MobileNetV2, MnasNet), whose
// expansion channels are the ones the method prunes.
//
// Run one after the other, the depthwise layer reads and writes the block's largest
// tensor (the expanded activations) and the 1x1 projection reads it again; here it is
// read once and never written.  A work-group owns an 8 x 8 block of output pixels of one
// image and MT projection filters.  Per chunk of expanded channels it stages the
// ((8-1)s+k)^2 input patch, the k*k depthwise weights and the [MT][chunk] slice of the
// projection weights in LDS; every thread then computes depthwise outputs (one 16-byte
// channel vector of one pixel per item, fp32 arithmetic) into an LDS tile laid out like
// the B operand of the dense kernels, and the four wavefronts multiply that tile with the
// projection slice on the matrix cores.  The channel loop is the reduction of the 1x1
// layer; bias, shortcut add and activation of the projection run in the epilogue.
// Values handed from the depthwise stage to the projection are rounded to the
// activation type, as they are when the depthwise layer stores its output.
//
// On small maps a layer has few pixel blocks (a 14x14 map at batch 64: 256, one per compute
// unit) and a long channel loop whose steps (global load -> LDS -> depthwise -> LDS ->
// MFMA) wait for each other.  KS > 1 puts KS groups of four wavefronts on one pixel block:
// group g takes chunks g, g + KS, ... with LDS buffers of its own, so the steps of KS chunks
// overlap; the groups' sums meet in LDS at the end, in group order.
#pragma once
#include "conv_nhwc_kernel.hpp"

namespace cprune {

template <int K, int S, int MB, int KQ, int KS>
constexpr int dwproj_lds_bytes() {
  constexpr int PH = 7 * S + K, ROW = 64 * KQ + 16;
  return KS * ((PH * PH + 64 + MB * 16) * ROW + K * K * 64 * KQ) + (KS > 1 ? MB * 4096 : 0);
}

template <typename T, int K, int S, int MB, int KQ, int KS>
__global__ __launch_bounds__(256 * KS) void dwproj_kernel(DwProjArgs a) {
  constexpr int NT = 256;                  // threads of one group
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;             // elements per 16-byte quad
  constexpr int CC = 4 * EPI * KQ;         // expanded channels per chunk
  constexpr int NQ = 4 * KQ;               // quads per pixel per chunk
  constexpr int TH = 8, TW = 8, PT = 64;
  constexpr int MT = MB * 16;
  constexpr int PH = (TH - 1) * S + K, PW = (TW - 1) * S + K;
  constexpr int NPATCH = PH * PW;
  constexpr int ROW = 64 * KQ + 16;        // bytes per LDS row (chunk + pad)
  constexpr int NI_IN = (NPATCH * NQ + NT - 1) / NT;
  constexpr int NI_A = (MT * NQ + NT - 1) / NT;
  constexpr int NI_DW = (PT * NQ) / NT;    // depthwise items (pixel, quad) per thread
  static_assert((PT * NQ) % NT == 0 && K * K * NQ <= NT, "item counts");
  constexpr int GROUP = NPATCH * ROW + PT * ROW + MT * ROW + K * K * 64 * KQ;   // LDS bytes of one group
  static_assert(dwproj_lds_bytes<K, S, MB, KQ, KS>() <= 160 * 1024, "LDS budget");

  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int t = threadIdx.x & (NT - 1);
  const int kgrp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
  unsigned char* sIn = lds + kgrp * GROUP;
  unsigned char* sB = sIn + NPATCH * ROW;
  unsigned char* sA = sB + PT * ROW;
  unsigned char* sW = sA + MT * ROW;

  const int lane = t & 63;
  const int wave = t >> 6;
  const int r = lane & 15, g4 = lane >> 4;

  int tile;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    tile = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  const int tile_m = tile % a.tiles_m;
  int rest = tile / a.tiles_m;
  const int tx0 = (rest % a.tiles_x) * TW;
  rest /= a.tiles_x;
  const int ty0 = (rest % a.tiles_y) * TH;
  const int n = rest / a.tiles_y;
  const int o0 = tile_m * MT;

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t pr = make_rsrc(a.wp, a.wp_bytes);
  const __amdgpu_buffer_rsrc_t dr = make_rsrc(a.wdw, a.wdw_bytes);

  // ---- staging items ----
  unsigned in_off[NI_IN];
  int in_lds[NI_IN], in_q[NI_IN];
#pragma unroll
  for (int j = 0; j < NI_IN; ++j) {
    const int idx = t + NT * j;
    const int q = idx % NQ, pp = idx / NQ;
    const bool item = pp < NPATCH;
    const int py = pp / PW, px = pp - py * PW;
    const int iy = ty0 * S - a.pad + py, ix = tx0 * S - a.pad + px;
    const bool inside = item && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
    in_off[j] = inside ? (unsigned)(((n * a.H + iy) * a.W + ix) * a.Cpe + q * EPI) * ES : kOutOfRange;
    in_lds[j] = item ? pp * ROW + q * 16 : -1;
    in_q[j] = q;
  }
  unsigned a_off[NI_A];
  int a_lds[NI_A], a_q[NI_A];
#pragma unroll
  for (int j = 0; j < NI_A; ++j) {
    const int idx = t + NT * j;
    const int q = idx % NQ, m = idx / NQ;
    const bool item = m < MT;
    const int o = o0 + m;
    a_off[j] = (item && o < a.O) ? (unsigned)(o * a.Cpe + q * EPI) * ES : kOutOfRange;
    a_lds[j] = item ? m * ROW + q * 16 : -1;
    a_q[j] = q;
  }
  // depthwise weights: one (tap, quad) item for the first K * K * NQ threads
  const bool w_item = t < K * K * NQ;
  const int w_q = t % NQ, w_tap = t / NQ;
  const unsigned w_off = w_item ? (unsigned)(w_tap * a.Cpe + w_q * EPI) * ES : kOutOfRange;
  const int w_lds = (w_tap * NQ + w_q) * 16;

  uint4 inreg[NI_IN], areg[NI_A], wreg;
  float bd_n[NI_DW][EPI];   // the chunk's depthwise biases travel with its weights, one chunk ahead of their use
  auto gload = [&](int c0) {
    const unsigned soff = (unsigned)(c0 * ES);
#pragma unroll
    for (int j = 0; j < NI_DW; ++j)
#pragma unroll
      for (int e = 0; e < EPI; ++e) {
        const int ch = c0 + ((t + NT * j) % NQ) * EPI + e;
        bd_n[j][e] = (a.bdw && ch < a.Ce) ? a.bdw[ch] : 0.0f;
      }
#pragma unroll
    for (int j = 0; j < NI_A; ++j) {
      const unsigned inval = (unsigned)(c0 + a_q[j] * EPI >= a.Cpe) << 31;
      areg[j] = load_b128(pr, a_off[j] | inval, soff);
    }
#pragma unroll
    for (int j = 0; j < NI_IN; ++j) {
      const unsigned inval = (unsigned)(c0 + in_q[j] * EPI >= a.Cpe) << 31;
      inreg[j] = load_b128(xr, in_off[j] | inval, soff);
    }
    const unsigned winval = (unsigned)(c0 + w_q * EPI >= a.Cpe) << 31;
    wreg = load_b128(dr, w_off | winval, soff);
  };
  auto lds_store = [&]() {
#pragma unroll
    for (int j = 0; j < NI_A; ++j)
      if (a_lds[j] >= 0) *(uint4*)&sA[a_lds[j]] = areg[j];
#pragma unroll
    for (int j = 0; j < NI_IN; ++j)
      if (in_lds[j] >= 0) *(uint4*)&sIn[in_lds[j]] = inreg[j];
    if (w_item) *(uint4*)&sW[w_lds] = wreg;
  };

  // ---- depthwise items of this thread: (pixel, quad) -> where its window starts ----
  int dw_in[NI_DW], dw_out[NI_DW], dw_q[NI_DW];
#pragma unroll
  for (int j = 0; j < NI_DW; ++j) {
    const int idx = t + NT * j;
    const int q = idx % NQ, p = idx / NQ;
    const int ty = p / TW, tx = p % TW;
    dw_in[j] = ((ty * S) * PW + tx * S) * ROW + q * 16;
    dw_out[j] = p * ROW + q * 16;
    dw_q[j] = q;
  }

  // ---- MFMA fragments ----
  const int b_frag = (wave * 16 + r) * ROW + g4 * 16;
  const int a_frag = r * ROW + g4 * 16;
  float4_t acc[MB][1];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i][0] = (float4_t){0.f, 0.f, 0.f, 0.f};

  int mb_count = (a.O - o0 + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;

  // group g takes chunks g, g + KS, ...: every group runs the same number of steps (a step past the last
  // chunk loads zeros), so the barriers match
  const int nchunk = (a.Cpe + CC - 1) / CC;
  const int nstep = (nchunk + KS - 1) / KS;
  auto main_loop = [&](auto mbc_tag) {
    constexpr int MBC = decltype(mbc_tag)::value;
    gload(kgrp * CC);
    for (int step = 0; step < nstep; ++step) {
      const int c = step * KS + kgrp;
      __syncthreads();              // previous chunk's MFMAs have read sA / sB, its depthwise pass sIn / sW
      lds_store();
      float bd[NI_DW][EPI];
#pragma unroll
      for (int j = 0; j < NI_DW; ++j)
#pragma unroll
        for (int e = 0; e < EPI; ++e) bd[j][e] = bd_n[j][e];
      __syncthreads();
      if (step + 1 < nstep) gload((c + KS) * CC);
      // depthwise: k x k window over the staged patch, fp32, bias, activation, rounded to T
#pragma unroll
      for (int j = 0; j < NI_DW; ++j) {
        float s[EPI];
#pragma unroll
        for (int e = 0; e < EPI; ++e) s[e] = 0.0f;
#pragma unroll
        for (int u = 0; u < K; ++u)
#pragma unroll
          for (int v = 0; v < K; ++v) {
            const uint4 xi = *(const uint4*)&sIn[dw_in[j] + (u * PW + v) * ROW];
            const uint4 wi = *(const uint4*)&sW[((u * K + v) * NQ + dw_q[j]) * 16];
            const T* xe = reinterpret_cast<const T*>(&xi);
            const T* we = reinterpret_cast<const T*>(&wi);
#pragma unroll
            for (int e = 0; e < EPI; ++e) s[e] += (float)xe[e] * (float)we[e];
          }
        uint4 o;
        T* oe = reinterpret_cast<T*>(&o);
#pragma unroll
        for (int e = 0; e < EPI; ++e) oe[e] = (T)apply_act(s[e] + bd[j][e], a.act_dw);
        *(uint4*)&sB[dw_out[j]] = o;
      }
      __syncthreads();
      // projection: the chunk is KQ rounds of the 1x1 layer's reduction
#pragma unroll
      for (int q4 = 0; q4 < KQ; ++q4) {
        uint4 af[MB], bf[1];
        bf[0] = *(const uint4*)&sB[b_frag + q4 * 64];
#pragma unroll
        for (int i = 0; i < MBC; ++i) af[i] = *(const uint4*)&sA[a_frag + i * 16 * ROW + q4 * 64];
        mma_slab<T, MBC, 1, MB>(af, bf, acc);
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

  if constexpr (KS > 1) {
    // the other groups hand their sums over one after the other through one exchange tile
    float4_t* xch = (float4_t*)(lds + KS * GROUP) + (size_t)wave * (MB * 64) + lane;
    for (int g = 1; g < KS; ++g) {
      __syncthreads();
      if (kgrp == g) {
#pragma unroll
        for (int i = 0; i < MB; ++i) xch[i * 64] = acc[i][0];
      }
      __syncthreads();
      if (kgrp == 0) {
#pragma unroll
        for (int i = 0; i < MB; ++i) acc[i][0] += xch[i * 64];
      }
    }
    if (kgrp != 0) return;
  }

  // ---- epilogue of the projection ----
  ConvArgs e;
  e.bias = a.bp; e.res = a.res; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act_out; e.vec_out = a.vec_out;
  const int pix = wave * 16 + r;
  const int oy = ty0 + pix / TW, ox = tx0 + pix % TW;
  if (oy < a.Ho && ox < a.Wo) {
    const int p = (n * a.Ho + oy) * a.Wo + ox;
#pragma unroll
    for (int i = 0; i < MB; ++i) nhwc_store4<T>(e, acc[i][0], p, o0 + i * 16 + 4 * g4);
  }
}

// Instantiations: k in {3, 5}, stride in {1, 2}, MB in {2, 4, 8} (tile of 32 / 64 / 128 filters), KS in {1, 2, 4}
// (4 only for the 3x3 window at stride 1: the 5x5 one needs more registers than 16 wavefronts leave, the
// stride-2 patch more LDS than four groups leave)
template <typename T>
inline int launch_dwproj(int k, int stride, int mb, int ks, dim3 grid, hipStream_t s, const DwProjArgs& a) {
#define CPRUNE_DWP(K_, S_, MB_, KS_)                                                                       \
  if (k == K_ && stride == S_ && mb == MB_ && ks == KS_) {                                                 \
    constexpr int lds = dwproj_lds_bytes<K_, S_, MB_, 1, KS_>();                                           \
    static bool raised = false;   /* more than the default 64 KiB of LDS has to be asked for once */       \
    if (lds > 65536 && !raised) {                                                                          \
      CPRUNE_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&dwproj_kernel<T, K_, S_, MB_, 1, KS_>), \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));         \
      raised = true;                                                                                       \
    }                                                                                                      \
    hipLaunchKernelGGL((dwproj_kernel<T, K_, S_, MB_, 1, KS_>), grid, dim3(256 * KS_), lds, s, a);         \
    return CPRUNE_OK;                                                                                      \
  }
#define CPRUNE_DWP3(K_, S_, KS_) CPRUNE_DWP(K_, S_, 2, KS_) CPRUNE_DWP(K_, S_, 4, KS_) CPRUNE_DWP(K_, S_, 8, KS_)
  CPRUNE_DWP3(3, 1, 1) CPRUNE_DWP3(3, 1, 2) CPRUNE_DWP3(3, 1, 4)
  CPRUNE_DWP3(3, 2, 1) CPRUNE_DWP3(3, 2, 2)
  CPRUNE_DWP3(5, 1, 1) CPRUNE_DWP3(5, 1, 2)
  CPRUNE_DWP3(5, 2, 1) CPRUNE_DWP3(5, 2, 2)
#undef CPRUNE_DWP3
#undef CPRUNE_DWP
  return CPRUNE_ERR_UNSUPPORTED;
}

}  // namespace cprune
