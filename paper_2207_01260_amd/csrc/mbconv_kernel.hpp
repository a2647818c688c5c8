// A whole inverted-residual block (MobileNetV2, MnasNet) in one kernel: 1x1 expansion (+ bias
// + activation), depthwise k x k (+ bias + activation) and 1x1 projection (+ bias + shortcut
// + activation).  The expansion channels are the ones the method prunes, and the expanded
// activations are the block's largest tensor by far (several times its input and output): run
// layer by layer they are written once and read twice; here they never leave the compute unit.
//
// A work-group owns an 8 x 8 block of output pixels of one image and all projection filters.
// It stages the ((8-1)s+k)^2 input patch once, all input channels (the expansion's whole
// reduction), and then walks over the expanded channels in chunks of 64 bytes per pixel:
//   1. expansion of the chunk's channels at every patch pixel on the matrix cores (weights x
//      patch), bias, activation, zero at pixels outside the image (they are the depthwise
//      layer's padding), rounded to the activation type -> LDS tile [patch pixel][chunk];
//   2. depthwise window over that tile, fp32 arithmetic, bias, activation, rounded -> LDS tile
//      [output pixel][chunk], laid out as the B operand of the projection;
//   3. projection: the chunk is one 64-byte round of the 1x1 layer's reduction.
// The halo of the patch is expanded again by the neighbouring work-groups ((8+k-1)^2 / 64 of
// the expansion's multiply-adds at stride 1, (15+k)^2 / 256 at stride 2): matrix-core work
// that is cheap next to the memory traffic it replaces.  Weights of the next chunk travel to
// registers during steps 1 and 2 and are stored into the other half of a double buffer
// before the barrier that separates steps 2 and 3; two barriers per chunk.
//
// Same MFMA blocks, lane layout and k-permutation as the other dense kernels.
#pragma once
#include "conv_nhwc_kernel.hpp"

namespace cprune {

template <typename T, int K, int S, int MB>
__global__ __launch_bounds__(256) void mbconv_kernel(MbConvArgs a) {
  constexpr int NT = 256;
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;             // elements per 16-byte quad
  constexpr int CC = 4 * EPI;              // expanded channels per chunk (64 bytes per pixel)
  constexpr int MBE = CC / 16;             // 16-row MFMA blocks of the expansion per chunk
  constexpr int TW = 8;
  constexpr int MT = MB * 16;
  constexpr int PH = 7 * S + K, PW = PH;
  constexpr int NPATCH = PH * PW;
  constexpr int NPATCHP = (NPATCH + 31) / 32 * 32;
  constexpr int NPAIR = NPATCHP / 32;      // pairs of 16-pixel blocks the expansion walks over
  constexpr int ROW = 64 + 16;             // bytes per LDS row of the chunk tiles
  constexpr int NI_A = (MT * 4 + NT - 1) / NT;
  constexpr int NWE = 2;                   // expansion-weight quads per thread and chunk (host checks CC * xq <= 512)
  static_assert(K * K * 4 <= NT, "depthwise weight items");

  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  unsigned char* sX = lds;
  unsigned char* sWe = lds + a.off_we;
  unsigned char* sE = lds + a.off_e;
  unsigned char* sB = lds + a.off_b;
  unsigned char* sA = lds + a.off_a;
  unsigned char* sW = lds + a.off_w;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int r = lane & 15, g4 = lane >> 4;

  int tile;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    tile = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  const int tx0 = (tile % a.tiles_x) * TW;
  int rest = tile / a.tiles_x;
  const int ty0 = (rest % a.tiles_y) * 8;
  const int n = rest / a.tiles_y;
  const int iy0 = ty0 * S - a.pad, ix0 = tx0 * S - a.pad;

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t er = make_rsrc(a.we, a.we_bytes);
  const __amdgpu_buffer_rsrc_t pr = make_rsrc(a.wp, a.wp_bytes);
  const __amdgpu_buffer_rsrc_t dr = make_rsrc(a.wdw, a.wdw_bytes);

  const int XQ = a.xq;
  const int XROW = XQ * 16 + 16;
  const int XR = XQ >> 2;                  // 64-byte rounds of the expansion's reduction

  // ---- the input patch, every input channel, once (eight loads in flight per thread) ----
  auto stage_patch = [&]() {
    constexpr int U = 8;
    const int total = NPATCHP * XQ;
    for (int base = t; base < total; base += NT * U) {
      uint4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = base + u * NT;
        const int pp = (int)fast_div((unsigned)idx, a.magic_xq);
        const int q = idx - pp * XQ;
        const int py = pp / PW, px = pp - py * PW;
        const int iy = iy0 + py, ix = ix0 + px;
        const bool inside = pp < NPATCH && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W && q * EPI < a.Cpi;
        const unsigned off = inside ? (unsigned)(((n * a.H + iy) * a.W + ix) * a.Cpi + q * EPI) * ES : kOutOfRange;
        v[u] = load_b128(xr, off, 0);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = base + u * NT;
        if (idx < total) {
          const int pp = (int)fast_div((unsigned)idx, a.magic_xq);
          *(uint4*)&sX[pp * XROW + (idx - pp * XQ) * 16] = v[u];
        }
      }
    }
  };

  // ---- weight staging items ----
  unsigned we_off[NWE];
  int we_lds[NWE], we_e[NWE];
#pragma unroll
  for (int j = 0; j < NWE; ++j) {
    const int idx = t + NT * j;
    const int e = (int)fast_div((unsigned)idx, a.magic_xq);
    const int q = idx - e * XQ;
    const bool item = e < CC;
    we_off[j] = (item && q * EPI < a.Cpi) ? (unsigned)(e * a.Cpi + q * EPI) * ES : kOutOfRange;
    we_lds[j] = item ? e * XROW + q * 16 : -1;
    we_e[j] = e;
  }
  unsigned a_off[NI_A];
  int a_lds[NI_A], a_q[NI_A];
#pragma unroll
  for (int j = 0; j < NI_A; ++j) {
    const int idx = t + NT * j;
    const int q = idx & 3, m = idx >> 2;
    const bool item = m < MT;
    a_off[j] = (item && m < a.O) ? (unsigned)(m * a.Cpe + q * EPI) * ES : kOutOfRange;
    a_lds[j] = item ? m * ROW + q * 16 : -1;
    a_q[j] = q;
  }
  const bool w_item = t < K * K * 4;
  const int w_q = t & 3, w_tap = t >> 2;
  const unsigned w_off = w_item ? (unsigned)(w_tap * a.Cpe + w_q * EPI) * ES : kOutOfRange;
  const int w_lds = (w_tap * 4 + w_q) * 16;

  uint4 wereg[NWE], areg[NI_A], wreg;
  auto gload = [&](int c0) {   // c0: first expanded channel of the chunk
#pragma unroll
    for (int j = 0; j < NWE; ++j) {
      // rows of the chunk start at channel c0; rows past the last expanded channel read as zero
      const unsigned inval = (unsigned)(c0 + we_e[j] >= a.Ce) << 31;
      wereg[j] = load_b128(er, we_off[j] | inval, (unsigned)(c0 * a.Cpi * ES));
    }
    const unsigned soff = (unsigned)(c0 * ES);
#pragma unroll
    for (int j = 0; j < NI_A; ++j) {
      const unsigned inval = (unsigned)(c0 + a_q[j] * EPI >= a.Cpe) << 31;
      areg[j] = load_b128(pr, a_off[j] | inval, soff);
    }
    const unsigned winval = (unsigned)(c0 + w_q * EPI >= a.Cpe) << 31;
    wreg = load_b128(dr, w_off | winval, soff);
  };
  auto lds_store = [&](int buf) {
#pragma unroll
    for (int j = 0; j < NWE; ++j)
      if (we_lds[j] >= 0) *(uint4*)&sWe[buf * CC * XROW + we_lds[j]] = wereg[j];
#pragma unroll
    for (int j = 0; j < NI_A; ++j)
      if (a_lds[j] >= 0) *(uint4*)&sA[buf * MT * ROW + a_lds[j]] = areg[j];
    if (w_item) *(uint4*)&sW[buf * K * K * 64 + w_lds] = wreg;
  };

  // ---- expansion: which patch pixels this lane's columns are, and whether they lie in the image ----
  // (pair p of pixel blocks: pixels 32p + 16j + r, j = 0, 1; wavefront w takes pairs w, w + 4, ...)
  // ---- depthwise item of this thread: (output pixel, quad) ----
  const int dq = t & 3, dp = t >> 2;
  const int dw_in = (((dp / TW) * S) * PW + (dp % TW) * S) * ROW + dq * 16;
  const int dw_out = dp * ROW + dq * 16;

  // ---- projection fragments ----
  const int b_frag = (wave * 16 + r) * ROW + g4 * 16;
  const int a_frag = r * ROW + g4 * 16;
  float4_t acc[MB][1];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i][0] = (float4_t){0.f, 0.f, 0.f, 0.f};
  int mb_count = (a.O + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;

  const int nchunk = (a.Cpe + CC - 1) / CC;
  gload(0);
  stage_patch();
  lds_store(0);
  __syncthreads();                 // patch and the first chunk's weights are in LDS

  auto main_loop = [&](auto mbc_tag) {
    constexpr int MBC = decltype(mbc_tag)::value;
    for (int c = 0; c < nchunk; ++c) {
      const int buf = c & 1;
      const int c0 = c * CC;
      if (c + 1 < nchunk) gload(c0 + CC);

      // 1. expansion of the chunk at every patch pixel
      float4_t eb[MBE];
#pragma unroll
      for (int i = 0; i < MBE; ++i) {
        const int ch = c0 + i * 16 + 4 * g4;
#pragma unroll
        for (int v = 0; v < 4; ++v) eb[i][v] = (a.be && ch + v < a.Ce) ? a.be[ch + v] : 0.0f;
      }
      const unsigned char* wbuf = sWe + buf * CC * XROW;
      for (int pair = wave; pair < NPAIR; pair += 4) {
        float4_t ea[MBE][2];
#pragma unroll
        for (int i = 0; i < MBE; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) ea[i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};
        const int xrow0 = (pair * 32 + r) * XROW + g4 * 16;
        for (int rnd = 0; rnd < XR; ++rnd) {
          uint4 af[MBE], bf[2];
#pragma unroll
          for (int j = 0; j < 2; ++j) bf[j] = *(const uint4*)&sX[xrow0 + j * 16 * XROW + rnd * 64];
#pragma unroll
          for (int i = 0; i < MBE; ++i) af[i] = *(const uint4*)&wbuf[(i * 16 + r) * XROW + g4 * 16 + rnd * 64];
          mma_slab<T, MBE, 2, MBE>(af, bf, ea);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int pp = pair * 32 + j * 16 + r;
          const int py = pp / PW, px = pp - py * PW;
          const bool inside = pp < NPATCH && (unsigned)(iy0 + py) < (unsigned)a.H && (unsigned)(ix0 + px) < (unsigned)a.W;
#pragma unroll
          for (int i = 0; i < MBE; ++i) {
            T h[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) h[v] = (T)(inside ? apply_act(ea[i][j][v] + eb[i][v], a.act_e) : 0.0f);
            unsigned char* dst = &sE[pp * ROW + (i * 16 + 4 * g4) * ES];
            if constexpr (ES == 4) *(uint4*)dst = *(const uint4*)h;
            else *(uint2*)dst = *(const uint2*)h;
          }
        }
      }
      __syncthreads();

      // 2. depthwise window over the expanded tile
      {
        float s[EPI];
#pragma unroll
        for (int e = 0; e < EPI; ++e) s[e] = 0.0f;
        const unsigned char* dwb = sW + buf * K * K * 64;
#pragma unroll
        for (int u = 0; u < K; ++u)
#pragma unroll
          for (int v = 0; v < K; ++v) {
            const uint4 xi = *(const uint4*)&sE[dw_in + (u * PW + v) * ROW];
            const uint4 wi = *(const uint4*)&dwb[((u * K + v) * 4 + dq) * 16];
            const T* xe = reinterpret_cast<const T*>(&xi);
            const T* wv = reinterpret_cast<const T*>(&wi);
#pragma unroll
            for (int e = 0; e < EPI; ++e) s[e] += (float)xe[e] * (float)wv[e];
          }
        uint4 o;
        T* oe = reinterpret_cast<T*>(&o);
#pragma unroll
        for (int e = 0; e < EPI; ++e) {
          const int ch = c0 + dq * EPI + e;
          const float b = (a.bdw && ch < a.Ce) ? a.bdw[ch] : 0.0f;
          oe[e] = (T)apply_act(s[e] + b, a.act_dw);
        }
        *(uint4*)&sB[dw_out] = o;
      }
      if (c + 1 < nchunk) lds_store(buf ^ 1);   // last read in chunk c - 1; visible after the barrier below
      __syncthreads();

      // 3. projection: one 64-byte round of its reduction
      {
        uint4 af[MB], bf[1];
        bf[0] = *(const uint4*)&sB[b_frag];
        const unsigned char* abuf = sA + buf * MT * ROW;
#pragma unroll
        for (int i = 0; i < MBC; ++i) af[i] = *(const uint4*)&abuf[a_frag + i * 16 * ROW];
        mma_slab<T, MBC, 1, MB>(af, bf, acc);
      }
      // the next chunk's expansion overwrites sE (read in step 2, behind a barrier) and its depthwise
      // step overwrites sB only after the barrier that ends its expansion
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

  // ---- epilogue of the projection ----
  ConvArgs e;
  e.bias = a.bp; e.res = a.res; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act_out; e.vec_out = a.vec_out;
  const int pix = wave * 16 + r;
  const int oy = ty0 + pix / TW, ox = tx0 + pix % TW;
  if (oy < a.Ho && ox < a.Wo) {
    const int p = (n * a.Ho + oy) * a.Wo + ox;
#pragma unroll
    for (int i = 0; i < MB; ++i) nhwc_store4<T>(e, acc[i][0], p, i * 16 + 4 * g4);
  }
}

// Instantiations: k in {3, 5}, stride in {1, 2}, MB in {2, 4, 8} (up to 32 / 64 / 128 projection filters)
template <typename T>
inline int launch_mbconv(int k, int stride, int mb, dim3 grid, size_t lds_bytes, hipStream_t s, const MbConvArgs& a) {
#define CPRUNE_MBC(K_, S_, MB_)                                                                         \
  if (k == K_ && stride == S_ && mb == MB_) {                                                           \
    static bool raised = false;   /* more than the default 64 KiB of LDS has to be asked for once */    \
    if (lds_bytes > 65536 && !raised) {                                                                 \
      CPRUNE_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&mbconv_kernel<T, K_, S_, MB_>), \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));      \
      raised = true;                                                                                    \
    }                                                                                                   \
    hipLaunchKernelGGL((mbconv_kernel<T, K_, S_, MB_>), grid, dim3(256), lds_bytes, s, a);              \
    return CPRUNE_OK;                                                                                   \
  }
  CPRUNE_MBC(3, 1, 2) CPRUNE_MBC(3, 1, 4) CPRUNE_MBC(3, 1, 8)
  CPRUNE_MBC(3, 2, 2) CPRUNE_MBC(3, 2, 4) CPRUNE_MBC(3, 2, 8)
  CPRUNE_MBC(5, 1, 2) CPRUNE_MBC(5, 1, 4) CPRUNE_MBC(5, 1, 8)
  CPRUNE_MBC(5, 2, 2) CPRUNE_MBC(5, 2, 4) CPRUNE_MBC(5, 2, 8)
#undef CPRUNE_MBC
  return CPRUNE_ERR_UNSUPPORTED;
}

}  // namespace cprune
