// Channels-last twin of the implicit-GEMM convolution kernel, used inside the
// network handle (Algorithm 1 of the paper: the pruned model run on the
// device).  Same tiling, MFMA blocks, slab pipeline, equal-run scheduling and
// fix-up as conv_igemm_kernel; what changes is how operands reach LDS.
//
// Activations are [n][h][w][cp] and weights [c_out][kh][kw][cp], with cp the
// channel count rounded up to one 16-byte vector (4 floats / 8 halves; the pad
// channels hold zeros).  The reduction index is k = (u, v, c), so for both
// operands 16 consecutive bytes of k are 16 consecutive bytes of memory: every
// staging item is one 128-bit buffer load and one 128-bit LDS store, and the
// im2col table holds one entry per 16-byte quad instead of one per element.  A
// pruned channel count that is not a multiple of the tile, or of 16, costs
// nothing extra: only the vector width is rounded.
#pragma once
#include "conv_kernel.hpp"

namespace cprune {

typedef unsigned int uint32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 load_b128(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  const uint32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <typename T, int WM, int WN, int MB, int NB, int KQ>
__global__ __launch_bounds__(256) void conv_nhwc_kernel(ConvArgs a) {
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;               // elements per 16-byte quad
  constexpr int KT = 4 * EPI * KQ;           // reduction elements per slab
  constexpr int ROW_BYTES = 64 * KQ + 16;
  constexpr int NQ = 4 * KQ;                 // quads per row
  constexpr int MT = WM * MB * 16;
  constexpr int PT = WN * NB * 16;
  constexpr int NIB = (PT * NQ + 255) / 256; // B items (pixel, quad) per thread
  constexpr int NIA = (MT * NQ + 255) / 256; // A items (filter, quad) per thread

  __shared__ __attribute__((aligned(16))) unsigned char sA[2][MT * ROW_BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char sB[2][PT * ROW_BYTES];
  __shared__ int tab_off[2][NQ];
  __shared__ unsigned tab_bits[2][NQ];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int r = lane & 15, g4 = lane >> 4;

  int g;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    g = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  int ub, ue;
  unit_range(a, g, ub, ue);

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t wr = make_rsrc(a.w, a.w_bytes);

  const int a_frag = (wm * MB * 16 + r) * ROW_BYTES + g4 * 16;
  const int b_frag = (wn * NB * 16 + r) * ROW_BYTES + g4 * 16;

  int seg = 0;
  for (int u = ub; u < ue; ++seg) {
    const int tile = u / a.slabs;
    const int s0 = u - tile * a.slabs;
    const int s1 = min(a.slabs, s0 + (ue - u));
    u += s1 - s0;
    const int nslab = s1 - s0;
    const int tile_m = tile % a.tiles_m;
    const int tile_p = tile / a.tiles_m;
    const int o0 = tile_m * MT;
    const int p0 = tile_p * PT;
    const int kbeg = s0 * KT;
    const int kend = min(a.K, s1 * KT);

    // ---- per-thread staging state for this tile ----
    int b_base[NIB];        // byte offset of the pixel's window origin (may be negative)
    unsigned b_mask[NIB];   // taps inside the image: bit u (rows), bit 8+v (columns)
    int b_lds[NIB];         // byte offset of the item's quad in a B buffer, -1 = none
    int b_q[NIB];
#pragma unroll
    for (int j = 0; j < NIB; ++j) {
      const int idx = t + 256 * j;
      const int pi = idx % PT, q = idx / PT;
      const bool item = idx < PT * NQ;
      unsigned pm = 0;
      int base = 0;
      const int p = p0 + pi;
      if (item && p < a.P) {
        const int n = p / a.HoWo;
        const int rem = p - n * a.HoWo;
        const int oy = rem / a.Wo;
        const int ox = rem - oy * a.Wo;
        const int iy0 = oy * a.stride - a.pad, ix0 = ox * a.stride - a.pad;
        base = ((n * a.H + iy0) * a.W + ix0) * a.Cp * ES;
        for (int uu = 0; uu < a.KH; ++uu)
          if ((unsigned)(iy0 + uu) < (unsigned)a.H) pm |= 1u << uu;
        for (int v = 0; v < a.KW; ++v)
          if ((unsigned)(ix0 + v) < (unsigned)a.W) pm |= 1u << (8 + v);
      }
      b_base[j] = base;
      b_mask[j] = pm;
      b_lds[j] = item ? pi * ROW_BYTES + q * 16 : -1;
      b_q[j] = item ? q : 0;
    }
    unsigned a_off[NIA];    // byte offset of (filter, kbeg + quad), kOutOfRange for filters past c_out
    int a_lds[NIA], a_q[NIA];
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      const int idx = t + 256 * j;
      const int m = idx / NQ, q = idx % NQ;
      const int o = o0 + m;
      const bool item = idx < MT * NQ;
      a_off[j] = (item && o < a.O) ? (unsigned)(o * a.K + kbeg + q * EPI) * ES : kOutOfRange;
      a_lds[j] = item ? m * ROW_BYTES + q * 16 : -1;
      a_q[j] = q;
    }

    auto write_table = [&](int slab, int slot) {
      if (t < NQ) {
        const int k = kbeg + slab * KT + t * EPI;
        int off = 0;
        unsigned bits = kOutOfRange;  // never satisfied by a pixel mask
        if (k < kend) {
          const unsigned tap = fast_div((unsigned)k, a.magic_cp);
          const unsigned c = (unsigned)k - tap * (unsigned)a.Cp;
          const unsigned uu = fast_div(tap, a.magic_kw);
          const unsigned v = tap - uu * (unsigned)a.KW;
          off = (int)((uu * (unsigned)a.W + v) * (unsigned)a.Cp + c) * ES;
          bits = (1u << uu) | (1u << (8 + v));
        }
        tab_off[slot][t] = off;
        tab_bits[slot][t] = bits;
      }
    };

    uint4 breg[NIB];
    uint4 areg[NIA];

    auto gload = [&](int slab, int slot) {
      const int k0 = kbeg + slab * KT;
      const unsigned soff = (unsigned)(slab * KT * ES);
#pragma unroll
      for (int j = 0; j < NIA; ++j) {
        const unsigned kinval = (unsigned)(k0 + a_q[j] * EPI >= kend) << 31;
        areg[j] = load_b128(wr, a_off[j] | kinval, soff);
      }
#pragma unroll
      for (int j = 0; j < NIB; ++j) {
        const int off = tab_off[slot][b_q[j]];
        const unsigned bits = tab_bits[slot][b_q[j]];
        breg[j] = load_b128(xr, (unsigned)(b_base[j] + off) | ((unsigned)((b_mask[j] & bits) != bits) << 31), 0);
      }
    };

    auto lds_store = [&](int buf) {
#pragma unroll
      for (int j = 0; j < NIA; ++j)
        if (a_lds[j] >= 0) *(uint4*)&sA[buf][a_lds[j]] = areg[j];
#pragma unroll
      for (int j = 0; j < NIB; ++j)
        if (b_lds[j] >= 0) *(uint4*)&sB[buf][b_lds[j]] = breg[j];
    };

    float4_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};

    int mb_count = (a.O - (o0 + wm * MB * 16) + 15) / 16;
    mb_count = mb_count < 0 ? 0 : (mb_count > MB ? MB : mb_count);

    auto main_loop = [&](auto mbc_tag) {
      constexpr int MBC = decltype(mbc_tag)::value;
      write_table(0, 0);
      __syncthreads();
      gload(0, 0);
      if (nslab > 1) write_table(1, 1);
      lds_store(0);
      __syncthreads();
      for (int s = 0; s < nslab; ++s) {
        const int buf = s & 1;
        uint4 af[MB], bf[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) bf[j] = *(const uint4*)&sB[buf][b_frag + j * 16 * ROW_BYTES];
#pragma unroll
        for (int i = 0; i < MBC; ++i) af[i] = *(const uint4*)&sA[buf][a_frag + i * 16 * ROW_BYTES];
        if (s + 1 < nslab) gload(s + 1, (s + 1) & 1);
        if (s + 2 < nslab) write_table(s + 2, s & 1);
        mma_slab<T, MBC, NB, MB>(af, bf, acc);
#pragma unroll
        for (int q4 = 1; q4 < KQ; ++q4) {
#pragma unroll
          for (int j = 0; j < NB; ++j) bf[j] = *(const uint4*)&sB[buf][b_frag + j * 16 * ROW_BYTES + q4 * 64];
#pragma unroll
          for (int i = 0; i < MBC; ++i) af[i] = *(const uint4*)&sA[buf][a_frag + i * 16 * ROW_BYTES + q4 * 64];
          mma_slab<T, MBC, NB, MB>(af, bf, acc);
        }
        if (s + 1 < nslab) lds_store(buf ^ 1);
        __syncthreads();
      }
    };
    switch (mb_count) {
#define CPRUNE_MBC_CASE(V) \
  case V: if constexpr (MB >= V) main_loop(std::integral_constant<int, V>{}); break;
      CPRUNE_MBC_CASE(0) CPRUNE_MBC_CASE(1) CPRUNE_MBC_CASE(2) CPRUNE_MBC_CASE(3) CPRUNE_MBC_CASE(4)
      CPRUNE_MBC_CASE(5) CPRUNE_MBC_CASE(6) CPRUNE_MBC_CASE(7) CPRUNE_MBC_CASE(8)
#undef CPRUNE_MBC_CASE
      default: break;
    }

    if (s0 == 0 && s1 == a.slabs) {
      const int m_wave = o0 + wm * MB * 16;
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int p = p0 + wn * NB * 16 + j * 16 + r;
        if (p >= a.P) continue;
#pragma unroll
        for (int i = 0; i < MB; ++i) nhwc_store4<T>(a, acc[i][j], p, m_wave + i * 16 + 4 * g4);
      }
    } else {
      float4_t* dst = (float4_t*)(a.partial + (size_t)(2 * g + (seg ? 1 : 0)) * (MT * PT)) + (size_t)wave * (MB * NB * 64) + lane;
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) dst[(i * NB + j) * 64] = acc[i][j];
    }
  }
}

// Fix-up of cut tiles, channels-last store (see conv_fixup_kernel).
template <typename T, int WM, int WN, int MB, int NB>
__global__ __launch_bounds__(256) void conv_nhwc_fixup_kernel(ConvArgs a) {
  constexpr int MT = WM * MB * 16, PT = WN * NB * 16;
  const int j = blockIdx.x;
  int ub, ue;
  unit_range(a, j, ub, ue);
  if (ub >= ue) return;
  const int tile = ub / a.slabs;
  const long first = (long)tile * a.slabs;
  if (ub == first || ue < first + a.slabs) return;
  const int g_lo = (int)(first / a.units_per_wg);
  const int g_hi = j;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int blk = blockIdx.y;
  const int bi = blk / NB, bj = blk % NB;
  const size_t elem = (size_t)wave * (MB * NB * 64) + (size_t)blk * 64 + lane;
  auto piece = [&](int g) -> const float4_t* {
    int gb, ge;
    unit_range(a, g, gb, ge);
    const int slot = 2 * g + ((gb / a.slabs == tile) ? 0 : 1);
    return (const float4_t*)(a.partial + (size_t)slot * (MT * PT)) + elem;
  };
  float4_t acc = (float4_t){0.f, 0.f, 0.f, 0.f};
  int g = g_lo;
  for (; g + 3 <= g_hi; g += 4) {
    const float4_t v0 = *piece(g), v1 = *piece(g + 1), v2 = *piece(g + 2), v3 = *piece(g + 3);
    acc += v0; acc += v1; acc += v2; acc += v3;
  }
  for (; g <= g_hi; ++g) acc += *piece(g);

  const int r = lane & 15, g4 = lane >> 4;
  const int tile_m = tile % a.tiles_m, tile_p = tile / a.tiles_m;
  const int p = tile_p * PT + wn * NB * 16 + bj * 16 + r;
  if (p >= a.P) return;
  nhwc_store4<T>(a, acc, p, tile_m * MT + wm * MB * 16 + bi * 16 + 4 * g4);
}

template <typename T>
inline void launch_tile_nhwc(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup) {
#define CPRUNE_TILE_CASE(ID, WM_, WN_, MB_, NB_, KQ_)                                                \
  case ID:                                                                                           \
    hipLaunchKernelGGL((conv_nhwc_kernel<T, WM_, WN_, MB_, NB_, KQ_>), grid, dim3(256), 0, s, a);    \
    if (fixup)                                                                                       \
      hipLaunchKernelGGL((conv_nhwc_fixup_kernel<T, WM_, WN_, MB_, NB_>), dim3(grid.x, MB_ * NB_), dim3(256), 0, s, a); \
    break;
  switch (tile) { CPRUNE_TILE_LIST(CPRUNE_TILE_CASE) }
#undef CPRUNE_TILE_CASE
}

void launch_conv_nhwc_f32(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup);
void launch_conv_nhwc_f16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup);
void launch_conv_nhwc_bf16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup);

}  // namespace cprune
