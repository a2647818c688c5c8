// Dense convolution as an implicit GEMM on the gfx950 matrix cores (device code).
//
// The subgraph of Section 3.4 of the paper (Conv2d + folded BN + ReLU) at the
// channel counts filter pruning leaves behind (Section 2.1): rows of the GEMM
// are the c_out surviving filters, columns the n*h_out*w_out output pixels, the
// reduction runs over k = (c, u, v) in the weights' own OIHW order.  Nothing is
// padded in HBM: tails in every dimension are zero-filled while staging into
// LDS and skipped in the epilogue; whole 16-row MFMA blocks past c_out are not
// issued at all (the main loop is compiled once per block count and the
// work-group picks its copy).
//
// One work-group = 4 wavefronts arranged WM x WN; a wavefront owns MB x NB
// accumulator blocks of 16x16 (v_mfma_f32_16x16x4_f32 for fp32 data,
// v_mfma_f32_16x16x32_{f16,bf16} for 16-bit data).  Per slab of the reduction
// (KT = 16 floats or 32 halves of k per row) the work-group stages an A tile
// [MT][KT] of weights and a B tile [PT][KT] of gathered input pixels into
// double-buffered LDS, rows k-contiguous, so each lane fetches its MFMA
// operands for the whole slab with one 16-byte LDS read per block.  The order
// in which k is consumed inside a slab is a permutation of the natural one
// (lane group g holds columns 4g..4g+3 of a 16-byte quad layout); A and B use
// the same permutation, which leaves the sum unchanged.
//
// Work is cut by slab iterations, not by tiles: the (tile, slab) pairs are laid
// out in one line, tile-major, and every work-group takes a contiguous run of
// units_per_wg of them.  With units_per_wg = slabs this is one tile per
// work-group; with fewer work-groups than tiles x slabs / units_per_wg the runs
// cut through tiles, so all compute units finish together whatever the channel
// and pixel counts are.  A tile that one work-group covers completely goes
// straight to the epilogue; the pieces of a cut tile are written as raw
// accumulators and summed, in run order, by conv_fixup_kernel (deterministic).
//
// The im2col gather is table-driven: for each k of a slab a small LDS table
// holds the input byte offset (c*H*W + u*W + v) and the tap bits (u, v); each
// staging thread keeps, per pixel it serves, a base offset and the mask of the
// taps that fall inside the image.  Loads are raw buffer loads: an element that
// is padding, past the end of k, or past the last pixel gets an offset beyond
// the buffer's size and reads as zero, without a branch.
#pragma once
#include "common.hpp"

#include <type_traits>

namespace cprune {

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

struct ConvArgs {
  const void* x;
  const void* w;
  const float* bias;
  const void* res;
  void* y;
  float* partial;  // [2 * work-groups][MT * PT] accumulator tiles of split output tiles
  int N, C, H, W, O, KH, KW, stride, pad, Ho, Wo;
  int K, P, HoWo, HW, KHW;
  unsigned magic_khw, magic_kw;  // ceil(2^32 / d), 0 when d == 1
  unsigned x_bytes, w_bytes;     // sizes of the x and w tensors (< 2^31)
  int act;
  int tiles_m, tiles_p;
  int Cp, Cop;        // channels-last kernels: channel stride of x / of y (elements)
  unsigned magic_cp;  // division by Cp
  int vec_out;        // channels-last: y may be written 4 channels at a time
  int nhwc_out = 0;   // NCHW-input kernel: y is channels-last [p][Cop] (the first layer of a network handle)
  int pool4 = 0;      // channels-last: rows 4c..4c+3 are the four positions of channel c of a 2x2 map;
                      // their maximum (behind bias and activation) is stored as y[p][c] (Cop = stride of y)
  int slabs;          // reduction slabs per output tile
  int units;          // tiles * slabs: the work, in slab iterations
  int units_per_wg;   // contiguous run of units each work-group takes
  unsigned magic_tp = 0;  // reduction-split kernel: division by tiles_p (exact while groups x tiles_p < 2^32)
  int w_packed = 0;   // reduction-split kernel: w is in fragment order, [16-row tile][round][lane][16 bytes]
};

constexpr unsigned kOutOfRange = 0x80000000u;  // beyond any buffer this kernel accepts

__device__ __forceinline__ unsigned fast_div(unsigned n, unsigned magic) {
  return magic ? __umulhi(n, magic) : n;
}

// Every activation here is a clamp: none = (-inf, +inf), ReLU = [0, +inf), ReLU6 = [0, 6].  The bounds are
// uniform and loop-invariant, so an element costs a max and a min; written as branches on `act` the
// compiler emitted a branch sequence per element (most of the time of a fused kernel's vector steps).
__device__ __forceinline__ float apply_act(float v, int act) {
  const float lo = act == CPRUNE_ACT_NONE ? -__builtin_inff() : 0.0f;
  const float hi = act == CPRUNE_ACT_RELU6 ? 6.0f : __builtin_inff();
  return fminf(fmaxf(v, lo), hi);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// bias[o .. o + 3] with zeros past the last filter (and for a null bias): four range-checked
// buffer loads, no branches
__device__ __forceinline__ float4_t load_bias4(const float* bias, int n_filters, int o) {
  const __amdgpu_buffer_rsrc_t br = make_rsrc(bias, bias ? (unsigned)n_filters * 4u : 0u);
  float4_t b;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    b[i] = __uint_as_float((unsigned)__builtin_amdgcn_raw_buffer_load_b32(br, (o + i) * 4, 0, 0));
  return b;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  typedef uint32_t raw_t;
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
  static __device__ __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0);
  }
};
template <> struct Elem<_Float16> {
  typedef uint16_t raw_t;
  static __device__ __forceinline__ float to_f32(_Float16 v) { return (float)v; }
  static __device__ __forceinline__ _Float16 from_f32(float v) { return (_Float16)v; }
  static __device__ __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_amdgcn_raw_buffer_load_b16(r, (int)voff, (int)soff, 0);
  }
};
template <> struct Elem<__bf16> {
  typedef uint16_t raw_t;
  static __device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }
  static __device__ __forceinline__ __bf16 from_f32(float v) { return (__bf16)v; }
  static __device__ __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_amdgcn_raw_buffer_load_b16(r, (int)voff, (int)soff, 0);
  }
};

// All MFMAs of one slab for MBC x NB blocks; consecutive instructions touch
// different accumulators.
template <typename T, int MBC, int NB, int MB>
__device__ __forceinline__ void mma_slab(const uint4 (&af)[MB], const uint4 (&bf)[NB], float4_t (&acc)[MB][NB]) {
  if constexpr (sizeof(T) == 4) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
#pragma unroll
      for (int i = 0; i < MBC; ++i) {
        const uint32_t av = e == 0 ? af[i].x : e == 1 ? af[i].y : e == 2 ? af[i].z : af[i].w;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const uint32_t bv = e == 0 ? bf[j].x : e == 1 ? bf[j].y : e == 2 ? bf[j].z : bf[j].w;
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(av), __uint_as_float(bv), acc[i][j], 0, 0, 0);
        }
      }
    }
  } else if constexpr (std::is_same<T, _Float16>::value) {
#pragma unroll
    for (int i = 0; i < MBC; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, af[i]),
                                                           __builtin_bit_cast(half8_t, bf[j]), acc[i][j], 0, 0, 0);
  } else {
#pragma unroll
    for (int i = 0; i < MBC; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, af[i]),
                                                            __builtin_bit_cast(bf16x8_t, bf[j]), acc[i][j], 0, 0, 0);
  }
}

template <int WM, int WN, int MB, int NB>
struct TileGeom {
  static constexpr int MT = WM * MB * 16;
  static constexpr int PT = WN * NB * 16;
};

// Where a work-group's run of units starts and ends.
__device__ __forceinline__ void unit_range(const ConvArgs& a, int g, int& ub, int& ue) {
  const long b = (long)g * a.units_per_wg;
  ub = (int)(b < a.units ? b : a.units);
  const long e = b + a.units_per_wg;
  ue = (int)(e < a.units ? e : a.units);
}

// bias + residual + activation + channels-last store of one 16x16 block column:
// a lane holds 4 consecutive channels of one pixel.
// (bias: the four values load_bias4 gives for o; kernels on short layers fetch them before their main loop,
// where the wait for them hides, and pass them in)
template <typename T>
__device__ __forceinline__ void nhwc_store4(const ConvArgs& a, const float4_t& acc, int p, int o, const float4_t& bias) {
  if (a.pool4) {
    if (o >= a.O) return;
    float m = apply_act(acc[0] + bias[0], a.act);
#pragma unroll
    for (int i = 1; i < 4; ++i) m = fmaxf(m, apply_act(acc[i] + bias[i], a.act));
    ((T*)a.y)[(size_t)p * a.Cop + (o >> 2)] = Elem<T>::from_f32(m);
    return;
  }
  if (o >= a.Cop) return;
  float v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = acc[i] + bias[i];
  const size_t off = (size_t)p * a.Cop + o;
  if (a.vec_out) {
    if (a.res) {
      if constexpr (sizeof(T) == 4) {
        const float4 rv = *(const float4*)((const float*)a.res + off);
        v[0] += rv.x; v[1] += rv.y; v[2] += rv.z; v[3] += rv.w;
      } else {
        const T* rp = (const T*)a.res + off;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] += Elem<T>::to_f32(rp[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = apply_act(v[i], a.act);
    if constexpr (sizeof(T) == 4) {
      *(float4*)((float*)a.y + off) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
      T h[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) h[i] = Elem<T>::from_f32(v[i]);
      *(uint2*)((T*)a.y + off) = *(const uint2*)h;
    }
  } else {
    // dense output whose channel stride is not a vector multiple (the logits)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (o + i < a.Cop) {
        float val = v[i];
        if (a.res) val += Elem<T>::to_f32(((const T*)a.res)[off + i]);
        ((T*)a.y)[off + i] = Elem<T>::from_f32(apply_act(val, a.act));
      }
    }
  }
}

template <typename T>
__device__ __forceinline__ void nhwc_store4(const ConvArgs& a, const float4_t& acc, int p, int o) {
  nhwc_store4<T>(a, acc, p, o, load_bias4(a.bias, a.O, o));
}

// bias + residual + activation + store of one wave's accumulators.
template <typename T, int WM, int WN, int MB, int NB>
__device__ __forceinline__ void conv_epilogue(const ConvArgs& a, const float4_t (&acc)[MB][NB], int tile_m,
                                              int tile_p, int wm, int wn, int r, int g4) {
  constexpr int MT = WM * MB * 16, PT = WN * NB * 16;
  T* __restrict__ yg = (T*)a.y;
  const T* __restrict__ rg = (const T*)a.res;
  const int m_wave = tile_m * MT + wm * MB * 16;
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int p = tile_p * PT + wn * NB * 16 + j * 16 + r;
    if (p >= a.P) continue;
    if (a.nhwc_out) {   // the pixel index is the same in both layouts; only the store differs
#pragma unroll
      for (int i = 0; i < MB; ++i) nhwc_store4<T>(a, acc[i][j], p, m_wave + i * 16 + 4 * g4);
      continue;
    }
    const int n = p / a.HoWo;
    const int rem = p - n * a.HoWo;
    const size_t pix = (size_t)n * a.O * a.HoWo + rem;
#pragma unroll
    for (int i = 0; i < MB; ++i) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int o = m_wave + i * 16 + 4 * g4 + v;
        if (o < a.O) {
          float val = acc[i][j][v] + (a.bias ? a.bias[o] : 0.0f);
          const size_t off = pix + (size_t)o * a.HoWo;
          if (rg) val += Elem<T>::to_f32(rg[off]);
          yg[off] = Elem<T>::from_f32(apply_act(val, a.act));
        }
      }
    }
  }
}

template <typename T, int WM, int WN, int MB, int NB, int KQ>
__global__ __launch_bounds__(256) void conv_igemm_kernel(ConvArgs a) {
  typedef typename Elem<T>::raw_t raw_t;
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;               // elements per 16-byte fragment
  constexpr int KT = 4 * EPI * KQ;           // reduction elements per slab (KQ MFMA rounds of 64 bytes)
  constexpr int ROW_BYTES = 64 * KQ + 16;    // k bytes per LDS row + 16 so rows rotate across banks
  constexpr int NQ = 4 * KQ;                 // 16-byte quads per row
  constexpr int MT = WM * MB * 16;
  constexpr int PT = WN * NB * 16;
  constexpr int NIB = (PT * NQ + 255) / 256; // B staging items (pixel, 16-byte quad) per thread
  constexpr int A_ROWS = 256 / KT;           // A rows staged per pass (KT threads along k)
  constexpr int NIA = (MT + A_ROWS - 1) / A_ROWS;

  __shared__ __attribute__((aligned(16))) unsigned char sA[2][MT * ROW_BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char sB[2][PT * ROW_BYTES];
  __shared__ __attribute__((aligned(16))) int tab_off[2][KT];
  __shared__ __attribute__((aligned(16))) unsigned tab_bits[2][KT];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int r = lane & 15, g4 = lane >> 4;

  // Work-groups are handed to the 8 XCDs round-robin; give each XCD a contiguous
  // stretch of the work so the groups sharing an L2 share input pixels and weights.
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

  const int a_k = t % KT;
  const int a_row0 = t / KT;
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
    int b_lds[NIB];         // byte offset of the item's 16-byte slot in a B buffer, -1 = none
    int b_tab[NIB];         // first table entry of the item's quad
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
        base = ((n * a.C * a.H + iy0) * a.W + ix0) * ES;
        for (int uu = 0; uu < a.KH; ++uu)
          if ((unsigned)(iy0 + uu) < (unsigned)a.H) pm |= 1u << uu;
        for (int v = 0; v < a.KW; ++v)
          if ((unsigned)(ix0 + v) < (unsigned)a.W) pm |= 1u << (8 + v);
      }
      b_base[j] = base;
      b_mask[j] = pm;
      b_lds[j] = item ? pi * ROW_BYTES + q * 16 : -1;
      b_tab[j] = item ? q * EPI : 0;
    }
    unsigned a_off[NIA];    // byte offset of (row, kbeg + a_k), kOutOfRange for rows past c_out
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      const int m = a_row0 + j * A_ROWS;
      const int o = o0 + m;
      a_off[j] = (m < MT && o < a.O) ? (unsigned)(o * a.K + kbeg + a_k) * ES : kOutOfRange;
    }

    auto write_table = [&](int slab, int slot) {
      if (t < KT) {
        const int k = kbeg + slab * KT + t;
        int off = 0;
        unsigned bits = kOutOfRange;  // never satisfied by a pixel mask
        if (k < kend) {
          const unsigned c = fast_div((unsigned)k, a.magic_khw);
          const unsigned rr = (unsigned)k - c * (unsigned)a.KHW;
          const unsigned uu = fast_div(rr, a.magic_kw);
          const unsigned v = rr - uu * (unsigned)a.KW;
          off = (int)(c * (unsigned)a.HW + uu * (unsigned)a.W + v) * ES;
          bits = (1u << uu) | (1u << (8 + v));
        }
        tab_off[slot][t] = off;
        tab_bits[slot][t] = bits;
      }
    };

    raw_t breg[NIB][EPI];
    raw_t areg[NIA];

    auto gload = [&](int slab, int slot) {
      const int k0 = kbeg + slab * KT;
      // offsets of elements that must read as zero get bit 31 set (arithmetic, not a
      // select of two loads: the loads stay unconditional and issue back to back)
      const unsigned kinval = (unsigned)(k0 + a_k >= kend) << 31;
      const unsigned soff = (unsigned)(slab * KT * ES);
#pragma unroll
      for (int j = 0; j < NIA; ++j) areg[j] = Elem<T>::load(wr, a_off[j] | kinval, soff);
#pragma unroll
      for (int j = 0; j < NIB; ++j) {
#pragma unroll
        for (int e4 = 0; e4 < EPI; e4 += 4) {
          const int4 offs = *(const int4*)&tab_off[slot][b_tab[j] + e4];
          const uint4 bits = *(const uint4*)&tab_bits[slot][b_tab[j] + e4];
          const unsigned m = b_mask[j];
          breg[j][e4 + 0] = Elem<T>::load(xr, (unsigned)(b_base[j] + offs.x) | ((unsigned)((m & bits.x) != bits.x) << 31), 0);
          breg[j][e4 + 1] = Elem<T>::load(xr, (unsigned)(b_base[j] + offs.y) | ((unsigned)((m & bits.y) != bits.y) << 31), 0);
          breg[j][e4 + 2] = Elem<T>::load(xr, (unsigned)(b_base[j] + offs.z) | ((unsigned)((m & bits.z) != bits.z) << 31), 0);
          breg[j][e4 + 3] = Elem<T>::load(xr, (unsigned)(b_base[j] + offs.w) | ((unsigned)((m & bits.w) != bits.w) << 31), 0);
        }
      }
    };

    auto lds_store = [&](int buf) {
#pragma unroll
      for (int j = 0; j < NIA; ++j) {
        const int m = a_row0 + j * A_ROWS;
        if (m < MT) *(raw_t*)&sA[buf][m * ROW_BYTES + a_k * ES] = areg[j];
      }
#pragma unroll
      for (int j = 0; j < NIB; ++j) {
        if (b_lds[j] >= 0) {
          uint4 pk;
          if constexpr (ES == 4) {
            pk = make_uint4(breg[j][0], breg[j][1], breg[j][2], breg[j][3]);
          } else {
            pk = make_uint4((uint32_t)breg[j][0] | ((uint32_t)breg[j][1] << 16),
                            (uint32_t)breg[j][2] | ((uint32_t)breg[j][3] << 16),
                            (uint32_t)breg[j][4] | ((uint32_t)breg[j][5] << 16),
                            (uint32_t)breg[j][6] | ((uint32_t)breg[j][7] << 16));
          }
          *(uint4*)&sB[buf][b_lds[j]] = pk;
        }
      }
    };

    // ---- accumulators ----
    float4_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = (float4_t){0.f, 0.f, 0.f, 0.f};

    // 16-row blocks of this wave that hold at least one real filter
    int mb_count = (a.O - (o0 + wm * MB * 16) + 15) / 16;
    mb_count = mb_count < 0 ? 0 : (mb_count > MB ? MB : mb_count);

    // ---- pipeline: the loop body is compiled for each possible block count ----
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
        // operands of the slab's first round first (their LDS latency overlaps the
        // address work below)
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

    // ---- epilogue: whole tile -> output; piece of a tile -> raw accumulators ----
    if (s0 == 0 && s1 == a.slabs) {
      conv_epilogue<T, WM, WN, MB, NB>(a, acc, tile_m, tile_p, wm, wn, r, g4);
    } else {
      // lane holds rows 4*g4..4*g4+3 of column r of each block; stored in that order
      float4_t* dst = (float4_t*)(a.partial + (size_t)(2 * g + (seg ? 1 : 0)) * (MT * PT)) + (size_t)wave * (MB * NB * 64) + lane;
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) dst[(i * NB + j) * 64] = acc[i][j];
    }
  }
}

// Sums the pieces of every output tile that was cut between work-groups, in the
// order of the runs, and applies the epilogue.  grid.x = one work-group per run,
// grid.y = one per accumulator block of the tile.  A run completes at most one
// cut tile: the one it starts in the middle of, if the run reaches that tile's
// last slab.  (Tiles a run starts at slab 0 are either whole, or completed by a
// later run.)  Pieces are fetched four at a time so their latencies overlap;
// the additions stay in run order, so the result does not depend on timing.
template <typename T, int WM, int WN, int MB, int NB>
__global__ __launch_bounds__(256) void conv_fixup_kernel(ConvArgs a) {
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
  const int blk = blockIdx.y;  // i * NB + jj
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

  // epilogue of one 16x16 block: lane holds rows 4*g4..4*g4+3 of column r
  const int r = lane & 15, g4 = lane >> 4;
  const int tile_m = tile % a.tiles_m, tile_p = tile / a.tiles_m;
  const int p = tile_p * PT + wn * NB * 16 + bj * 16 + r;
  if (p >= a.P) return;
  if (a.nhwc_out) {
    nhwc_store4<T>(a, acc, p, tile_m * MT + wm * MB * 16 + bi * 16 + 4 * g4);
    return;
  }
  const int n = p / a.HoWo;
  const int rem = p - n * a.HoWo;
  const size_t pix = (size_t)n * a.O * a.HoWo + rem;
  T* __restrict__ yg = (T*)a.y;
  const T* __restrict__ rg = (const T*)a.res;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int o = tile_m * MT + wm * MB * 16 + bi * 16 + 4 * g4 + v;
    if (o < a.O) {
      float val = acc[v] + (a.bias ? a.bias[o] : 0.0f);
      const size_t off = pix + (size_t)o * a.HoWo;
      if (rg) val += Elem<T>::to_f32(rg[off]);
      yg[off] = Elem<T>::from_f32(apply_act(val, a.act));
    }
  }
}

// Tile table shared by the launchers: id, wm, wn, mb, nb, kq.  Small tiles take deeper
// slabs (kq rounds of 64 bytes of k per barrier): their per-slab MFMA work is short
// against the latency of the loads that feed the next slab.
#define CPRUNE_TILE_LIST(X) \
  X(0, 1, 4, 4, 4, 1)  /* 64 x 256  */ \
  X(1, 2, 2, 4, 4, 1)  /* 128 x 128 */ \
  X(2, 1, 4, 8, 2, 1)  /* 128 x 128 */ \
  X(3, 1, 4, 2, 4, 1)  /* 32 x 256  */ \
  X(4, 1, 4, 4, 2, 1)  /* 64 x 128  */ \
  X(5, 1, 4, 4, 2, 2)  /* 64 x 128, deep */ \
  X(6, 1, 4, 3, 4, 1)  /* 48 x 256  */ \
  X(7, 1, 4, 1, 4, 1)  /* 16 x 256  */ \
  X(8, 1, 4, 2, 2, 2)  /* 32 x 128, deep */ \
  X(9, 1, 4, 1, 2, 2)  /* 16 x 128, deep */ \
  X(10, 1, 4, 4, 1, 1) /* 64 x 64   */ \
  X(11, 1, 4, 4, 1, 2) /* 64 x 64, deep */ \
  X(12, 1, 4, 2, 1, 4) /* 32 x 64, deep */ \
  X(13, 1, 4, 8, 1, 1) /* 128 x 64  */ \
  X(14, 1, 4, 8, 1, 2) /* 128 x 64, deep */ \
  X(15, 1, 4, 1, 1, 4) /* 16 x 64, deep */ \
  X(16, 1, 4, 6, 2, 1) /* 96 x 128  */ \
  X(17, 1, 4, 2, 1, 1) /* 32 x 64   */

constexpr int kNumTiles = 18;

template <typename T>
inline void launch_tile(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup) {
#define CPRUNE_TILE_CASE(ID, WM_, WN_, MB_, NB_, KQ_)                                                \
  case ID:                                                                                           \
    hipLaunchKernelGGL((conv_igemm_kernel<T, WM_, WN_, MB_, NB_, KQ_>), grid, dim3(256), 0, s, a);   \
    if (fixup)                                                                                       \
      hipLaunchKernelGGL((conv_fixup_kernel<T, WM_, WN_, MB_, NB_>), dim3(grid.x, MB_ * NB_), dim3(256), 0, s, a); \
    break;
  switch (tile) { CPRUNE_TILE_LIST(CPRUNE_TILE_CASE) }
#undef CPRUNE_TILE_CASE
}

// Per-dtype launch entry points, one translation unit each.
void launch_conv_f32(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup);
void launch_conv_f16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup);
void launch_conv_bf16(int tile, dim3 grid, hipStream_t s, const ConvArgs& a, bool fixup);

}  // namespace cprune
