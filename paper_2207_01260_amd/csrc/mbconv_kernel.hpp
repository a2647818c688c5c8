// A whole inverted-residual block (MobileNetV2, MnasNet) in one kernel: 1x1 expansion (+ bias
// + activation), depthwise k x k (+ bias + activation) and 1x1 projection (+ bias + shortcut
// + activation).  The expansion channels are the ones the method prunes, and the expanded
// activations are the block's largest tensor by far (several times its input and output): run
// layer by layer they are written once and read twice; here they never leave the compute unit.
//
// Work-groups are persistent: each loads ALL weights and biases of the three layers into LDS
// once (which is what limits the kernel to blocks whose weights fit beside the tiles) and then
// walks over 8 x 8 blocks of output pixels.  Per block it stages the ((8-1)s+k)^2 input patch,
// all input channels (the expansion's whole reduction), and goes over the expanded channels in
// chunks of 64 bytes per pixel:
//   1. expansion of the chunk's channels at every patch pixel on the matrix cores (weights x
//      patch), bias, activation, zero at pixels outside the image (they are the depthwise
//      layer's padding), rounded to the activation type -> LDS tile [patch pixel][chunk];
//   2. depthwise window over that tile, fp32 arithmetic, bias, activation, rounded -> LDS tile
//      [output pixel][chunk], laid out as the B operand of the projection;
//   3. projection: the chunk is one 64-byte round of the 1x1 layer's reduction.
// The three steps are software-pipelined over the chunks: between two barriers a wavefront runs
// step 1 of chunk p, step 2 of chunk p - 1 and step 3 of chunk p - 2 (the two LDS tiles are double
// buffers), so that every interval holds matrix-core work, vector work and LDS traffic that do not
// depend on each other; one barrier per chunk.  No global memory is touched inside the chunk loop
// except the next block's input patch, which travels to registers meanwhile.  The halo of the
// patch is expanded again by the neighbouring blocks ((8+k-1)^2 / 64 of the expansion's
// multiply-adds at stride 1, (15+k)^2 / 256 at stride 2): matrix-core work that is cheap next
// to the memory traffic it replaces.
//
// Same MFMA blocks, lane layout and k-permutation as the other dense kernels.
#pragma once
#include <atomic>
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
  constexpr int KK = K * K;
  constexpr int PH = 7 * S + K, PW = PH;
  constexpr int NPATCH = PH * PW;
  constexpr int NPATCHP = (NPATCH + 31) / 32 * 32;
  constexpr int NPAIR = NPATCHP / 32;      // pairs of 16-pixel blocks the expansion walks over
  constexpr int ROW = 64 + 16;             // bytes per LDS row of the chunk tiles
  constexpr int U = 4;                     // loads in flight per thread while staging
  constexpr int NPRE = 10;                 // 16-byte pieces of the next input patch a thread holds (host checks the fit)
  constexpr int SE = NPATCHP * ROW, SB = 64 * ROW;

  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  unsigned char* sX = lds;                       // [NPATCHP][XROW] input patch
  unsigned char* sE = lds + a.off_e;             // [2][NPATCHP][ROW] expanded chunk (double buffer)
  unsigned char* sB = lds + a.off_b;             // [2][64][ROW] depthwise output chunk (double buffer)
  unsigned char* sWe = lds + a.off_we;           // [nchunk * CC][XROW] expansion weights
  unsigned char* sA = lds + a.off_a;             // [nchunk][MT][ROW] projection weights, chunk-major
  unsigned char* sW = lds + a.off_w;             // [nchunk][K * K][64] depthwise weights, chunk-major
  float* sBe = (float*)(lds + a.off_bias);       // [nchunk * CC] expansion bias
  float* sBd = sBe + a.nchunk * CC;              // [nchunk * CC] depthwise bias

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int r = lane & 15, g4 = lane >> 4;

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t er = make_rsrc(a.we, a.we_bytes);
  const __amdgpu_buffer_rsrc_t pr = make_rsrc(a.wp, a.wp_bytes);
  const __amdgpu_buffer_rsrc_t dr = make_rsrc(a.wdw, a.wdw_bytes);

  const int XQ = a.xq;
  const int XROW = XQ * 16 + 16;
  const int XR = XQ >> 2;                  // 64-byte rounds of the expansion's reduction
  const int nchunk = a.nchunk;
  const int CeP = nchunk * CC;

  // ---- once per work-group: every weight and bias of the block ----
  // `count` 16-byte items, item idx read at byte offset src(idx) (kOutOfRange = zero) and stored at dst(idx)
  auto stage = [&](int count, __amdgpu_buffer_rsrc_t rs, unsigned char* base, auto src, auto dst) {
    for (int b0 = t; b0 < count; b0 += NT * U) {
      uint4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = load_b128(rs, src(b0 + u * NT), 0);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (b0 + u * NT < count) *(uint4*)&base[dst(b0 + u * NT)] = v[u];
    }
  };
  stage(CeP * XQ, er, sWe,
        [&](int idx) -> unsigned {
          const int e = (int)fast_div((unsigned)idx, a.magic_xq), q = idx - e * XQ;
          return (e < a.Ce && q * EPI < a.Cpi) ? (unsigned)(e * a.Cpi + q * EPI) * ES : kOutOfRange;
        },
        [&](int idx) -> int {
          const int e = (int)fast_div((unsigned)idx, a.magic_xq), q = idx - e * XQ;
          return e * XROW + q * 16;
        });
  stage(nchunk * MT * 4, pr, sA,
        [&](int idx) -> unsigned {
          const int q = idx & 3, m = (idx >> 2) % MT, c = (idx >> 2) / MT;
          const int ch = c * CC + q * EPI;
          return (c < nchunk && m < a.O && ch < a.Cpe) ? (unsigned)(m * a.Cpe + ch) * ES : kOutOfRange;
        },
        [&](int idx) -> int { return (idx >> 2) * ROW + (idx & 3) * 16; });
  stage(nchunk * KK * 4, dr, sW,
        [&](int idx) -> unsigned {
          const int q = idx & 3, tap = (idx >> 2) % KK, c = (idx >> 2) / KK;
          const int ch = c * CC + q * EPI;
          return (c < nchunk && ch < a.Cpe) ? (unsigned)(tap * a.Cpe + ch) * ES : kOutOfRange;
        },
        [&](int idx) -> int { return idx * 16; });
  for (int ch = t; ch < CeP; ch += NT) {
    sBe[ch] = (a.be && ch < a.Ce) ? a.be[ch] : 0.0f;
    sBd[ch] = (a.bdw && ch < a.Ce) ? a.bdw[ch] : 0.0f;
  }

  // ---- per-thread constants of the three steps ----
  const int dq = t & 3, dp = t >> 2;       // depthwise item: (output pixel, quad)
  const int dw_in = (((dp / TW) * S) * PW + (dp % TW) * S) * ROW + dq * 16;
  const int dw_out = dp * ROW + dq * 16;
  const int b_frag = (wave * 16 + r) * ROW + g4 * 16;
  const int a_frag = r * ROW + g4 * 16;
  int mb_count = (a.O + 15) / 16;
  mb_count = mb_count > MB ? MB : mb_count;
  ConvArgs e;
  e.bias = a.bp; e.res = a.res; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act_out; e.vec_out = a.vec_out;

  int worker;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    worker = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  const int ntiles = a.N * a.tiles_y * a.tiles_x;

  // the input patch of a block: piece j of this thread is item t + 256 * j of [NPATCHP][XQ]
  const int npieces = NPATCHP * XQ;
  uint4 pre[NPRE];
  auto load_patch = [&](int tile) {
    const int tx0 = (tile % a.tiles_x) * TW;
    int rest = tile / a.tiles_x;
    const int ty0 = (rest % a.tiles_y) * 8;
    const int n = rest / a.tiles_y;
    const int iy0 = ty0 * S - a.pad, ix0 = tx0 * S - a.pad;
#pragma unroll
    for (int j = 0; j < NPRE; ++j) {
      const int idx = t + NT * j;
      const int pp = (int)fast_div((unsigned)idx, a.magic_xq), q = idx - pp * XQ;
      const int py = pp / PW, px = pp - py * PW;
      const int iy = iy0 + py, ix = ix0 + px;
      const bool inside = idx < npieces && pp < NPATCH && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W &&
                          q * EPI < a.Cpi;
      pre[j] = load_b128(xr, inside ? (unsigned)(((n * a.H + iy) * a.W + ix) * a.Cpi + q * EPI) * ES : kOutOfRange, 0);
    }
  };
  auto store_patch = [&]() {
#pragma unroll
    for (int j = 0; j < NPRE; ++j) {
      const int idx = t + NT * j;
      if (idx < npieces) {
        const int pp = (int)fast_div((unsigned)idx, a.magic_xq), q = idx - pp * XQ;
        *(uint4*)&sX[pp * XROW + q * 16] = pre[j];
      }
    }
  };

  if (worker < ntiles) load_patch(worker);
  for (int tile = worker; tile < ntiles; tile += (int)gridDim.x) {
    const int tx0 = (tile % a.tiles_x) * TW;
    int rest = tile / a.tiles_x;
    const int ty0 = (rest % a.tiles_y) * 8;
    const int n = rest / a.tiles_y;
    const int iy0 = ty0 * S - a.pad, ix0 = tx0 * S - a.pad;

    __syncthreads();               // the previous block's readers of the patch are done
    store_patch();
    __syncthreads();               // patch (and, the first time, the weights) are in LDS
    if (tile + (int)gridDim.x < ntiles) load_patch(tile + (int)gridDim.x);

    float4_t acc[MB][1];
#pragma unroll
    for (int i = 0; i < MB; ++i) acc[i][0] = (float4_t){0.f, 0.f, 0.f, 0.f};

    // 1. expansion of chunk c at every patch pixel; wavefront w takes pixel-block pairs w, w + 4, ...
    auto expand = [&](int c, unsigned char* dstE) {
      const int c0 = c * CC;
      float4_t eb[MBE];
#pragma unroll
      for (int i = 0; i < MBE; ++i) eb[i] = *(const float4_t*)&sBe[c0 + i * 16 + 4 * g4];
      const unsigned char* wbuf = sWe + c0 * XROW;
      for (int pair = wave; pair < NPAIR; pair += 4) {
        float4_t ea[MBE][2];
#pragma unroll
        for (int i = 0; i < MBE; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) ea[i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};
        const int xrow0 = (pair * 32 + r) * XROW + g4 * 16;
        // operands of round rnd + 1 are fetched from LDS while round rnd is multiplied (two register sets)
        uint4 af0[MBE], bf0[2], af1[MBE], bf1[2];
        auto fetch = [&](int rnd, uint4 (&fa)[MBE], uint4 (&fb)[2]) {
#pragma unroll
          for (int j = 0; j < 2; ++j) fb[j] = *(const uint4*)&sX[xrow0 + j * 16 * XROW + rnd * 64];
#pragma unroll
          for (int i = 0; i < MBE; ++i) fa[i] = *(const uint4*)&wbuf[(i * 16 + r) * XROW + g4 * 16 + rnd * 64];
        };
        fetch(0, af0, bf0);
        for (int rnd = 0; rnd < XR; rnd += 2) {
          const bool second = rnd + 1 < XR;
          if (second) fetch(rnd + 1, af1, bf1);
          mma_slab<T, MBE, 2, MBE>(af0, bf0, ea);
          if (rnd + 2 < XR) fetch(rnd + 2, af0, bf0);
          if (second) mma_slab<T, MBE, 2, MBE>(af1, bf1, ea);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int pp = pair * 32 + j * 16 + r;
          const int py = pp / PW, px = pp - py * PW;
          const bool inside = pp < NPATCH && (unsigned)(iy0 + py) < (unsigned)a.H && (unsigned)(ix0 + px) < (unsigned)a.W;
          const float keep = inside ? 1.0f : 0.0f;   // a factor, not a branch: activations are finite
#pragma unroll
          for (int i = 0; i < MBE; ++i) {
            T h[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) h[v] = (T)(keep * apply_act(ea[i][j][v] + eb[i][v], a.act_e));
            unsigned char* dst = &dstE[pp * ROW + (i * 16 + 4 * g4) * ES];
            if constexpr (ES == 4) *(uint4*)dst = *(const uint4*)h;
            else *(uint2*)dst = *(const uint2*)h;
          }
        }
      }
    };
    // 2. depthwise window over the expanded tile of chunk c
    auto depthwise = [&](int c, const unsigned char* srcE, unsigned char* dstB) {
      float s[EPI];
#pragma unroll
      for (int q = 0; q < EPI; ++q) s[q] = 0.0f;
      const unsigned char* dwb = sW + c * KK * 64;
#pragma unroll
      for (int u = 0; u < K; ++u)
#pragma unroll
        for (int v = 0; v < K; ++v) {
          const uint4 xi = *(const uint4*)&srcE[dw_in + (u * PW + v) * ROW];
          const uint4 wi = *(const uint4*)&dwb[((u * K + v) * 4 + dq) * 16];
          const T* xe = reinterpret_cast<const T*>(&xi);
          const T* wv = reinterpret_cast<const T*>(&wi);
#pragma unroll
          for (int q = 0; q < EPI; ++q) s[q] += (float)xe[q] * (float)wv[q];
        }
      uint4 o;
      T* oe = reinterpret_cast<T*>(&o);
#pragma unroll
      for (int q4 = 0; q4 < EPI / 4; ++q4) {
        const float4_t bd = *(const float4_t*)&sBd[c * CC + dq * EPI + 4 * q4];
#pragma unroll
        for (int v = 0; v < 4; ++v) oe[4 * q4 + v] = (T)apply_act(s[4 * q4 + v] + bd[v], a.act_dw);
      }
      *(uint4*)&dstB[dw_out] = o;
    };

    auto main_loop = [&](auto mbc_tag) {
      constexpr int MBC = decltype(mbc_tag)::value;
      // interval p: expansion of chunk p into sE[p & 1] (last read by the depthwise step of chunk
      // p - 2, one interval ago), depthwise step of chunk p - 1 from sE[(p - 1) & 1] into
      // sB[(p - 1) & 1] (last read by the projection of chunk p - 3, one interval ago), projection
      // of chunk p - 2 from sB[p & 1] (written one interval ago)
      for (int p = 0; p < nchunk + 2; ++p) {
        if (p < nchunk) expand(p, sE + (p & 1) * SE);
        if (p >= 1 && p <= nchunk) depthwise(p - 1, sE + ((p - 1) & 1) * SE, sB + ((p - 1) & 1) * SB);
        if (p >= 2) {
          uint4 af[MB], bf[1];
          bf[0] = *(const uint4*)&sB[(p & 1) * SB + b_frag];
          const unsigned char* abuf = sA + (p - 2) * MT * ROW;
#pragma unroll
          for (int i = 0; i < MBC; ++i) af[i] = *(const uint4*)&abuf[a_frag + i * 16 * ROW];
          mma_slab<T, MBC, 1, MB>(af, bf, acc);
        }
        __syncthreads();
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
    const int pix = wave * 16 + r;
    const int oy = ty0 + pix / TW, ox = tx0 + pix % TW;
    if (oy < a.Ho && ox < a.Wo) {
      const int p = (n * a.Ho + oy) * a.Wo + ox;
#pragma unroll
      for (int i = 0; i < MB; ++i) nhwc_store4<T>(e, acc[i][0], p, i * 16 + 4 * g4);
    }
  }
}

// Instantiations: k in {3, 5}, stride in {1, 2}, MB in {2, 4, 8} (up to 32 / 64 / 128 projection filters)
template <typename T>
inline int launch_mbconv(int k, int stride, int mb, dim3 grid, size_t lds_bytes, hipStream_t s, const MbConvArgs& a) {
#define CPRUNE_MBC(K_, S_, MB_)                                                                         \
  if (k == K_ && stride == S_ && mb == MB_) {                                                           \
    static std::atomic<bool> raised{false};   /* more than the default 64 KiB of LDS has to be asked for once */ \
    if (lds_bytes > 65536 && !raised.load(std::memory_order_relaxed)) {                                       \
      CPRUNE_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&mbconv_kernel<T, K_, S_, MB_>), \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));      \
      raised.store(true, std::memory_order_relaxed);                                                          \
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
