// Dense convolution as an implicit GEMM on the gfx950 matrix cores.
//
// The subgraph of Section 3.4 of the paper (Conv2d + folded BN + ReLU) at the
// channel counts filter pruning leaves behind (Section 2.1): rows of the GEMM
// are the c_out surviving filters, columns the n*h_out*w_out output pixels, the
// reduction runs over k = (c, u, v) in the weights' own OIHW order.  Nothing is
// padded in HBM: tails in every dimension are zero-filled while staging into
// LDS and skipped in the epilogue; whole 16-row MFMA blocks past c_out are not
// issued at all.
//
// One work-group = 4 wavefronts arranged WM x WN; a wavefront owns MB x NB
// accumulator blocks of 16x16 (v_mfma_f32_16x16x4_f32 for fp32 data,
// v_mfma_f32_16x16x32_{f16,bf16} for 16-bit data).  Per slab of the reduction
// (KT = 16 floats or 32 halves of k per row) the work-group
// stages an A tile [MT][KT] of weights and a B tile [PT][KT] of gathered input
// pixels into double-buffered LDS, rows k-contiguous, so each lane fetches its
// MFMA operands for the whole slab with one 16-byte LDS read per block.  The
// order in which k is consumed inside a slab is a permutation of the natural
// one (lane group g holds columns 4g..4g+3); A and B use the same permutation,
// which leaves the sum unchanged.
//
// The im2col gather is table-driven: for each k of a slab a small LDS table
// holds the input offset (c*H*W + u*W + v) and the tap bits (u, v); each
// staging thread keeps, per pixel it serves, a base offset and the masks of the
// taps that fall inside the image, so one element costs an add, an and/compare
// and a predicated load.
#include "common.hpp"

namespace cprune {
namespace {

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

struct ConvArgs {
  const void* x;
  const void* w;
  const float* bias;
  const void* res;
  void* y;
  float* partial;  // [split_k][O][P] when split_k > 1
  int N, C, H, W, O, KH, KW, stride, pad, Ho, Wo;
  int K, P, HoWo, HW, KHW;
  unsigned magic_khw, magic_kw;  // ceil(2^32 / d), 0 when d == 1
  int act;
  int tiles_m;
  int split_k, k_per_split;
};

__device__ __forceinline__ unsigned fast_div(unsigned n, unsigned magic) {
  return magic ? __umulhi(n, magic) : n;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  typedef uint32_t raw_t;
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elem<_Float16> {
  typedef uint16_t raw_t;
  static __device__ __forceinline__ float to_f32(_Float16 v) { return (float)v; }
  static __device__ __forceinline__ _Float16 from_f32(float v) { return (_Float16)v; }
};
template <> struct Elem<__bf16> {
  typedef uint16_t raw_t;
  static __device__ __forceinline__ float to_f32(__bf16 v) { return (float)v; }
  static __device__ __forceinline__ __bf16 from_f32(float v) { return (__bf16)v; }
};

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == CPRUNE_ACT_RELU) return fmaxf(v, 0.0f);
  if (act == CPRUNE_ACT_RELU6) return fminf(fmaxf(v, 0.0f), 6.0f);
  return v;
}

// One slab's worth of MFMAs on a 16-byte A fragment and a 16-byte B fragment.
template <typename T>
__device__ __forceinline__ void mma_frag(const uint4& a, const uint4& b, float4_t& acc);

template <>
__device__ __forceinline__ void mma_frag<float>(const uint4& a, const uint4& b, float4_t& acc) {
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma_frag<_Float16>(const uint4& a, const uint4& b, float4_t& acc) {
  half8_t av = __builtin_bit_cast(half8_t, a);
  half8_t bv = __builtin_bit_cast(half8_t, b);
  acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma_frag<__bf16>(const uint4& a, const uint4& b, float4_t& acc) {
  bf16x8_t av = __builtin_bit_cast(bf16x8_t, a);
  bf16x8_t bv = __builtin_bit_cast(bf16x8_t, b);
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc, 0, 0, 0);
}

constexpr int ROW_BYTES = 80;  // 64 bytes of k per row + 16 bytes so rows rotate across LDS banks

template <typename T, int WM, int WN, int MB, int NB>
__global__ __launch_bounds__(256) void conv_igemm_kernel(ConvArgs a) {
  typedef typename Elem<T>::raw_t raw_t;
  constexpr int EPI = 16 / (int)sizeof(T);  // elements per 16-byte fragment
  constexpr int KT = 4 * EPI;               // reduction elements per slab
  constexpr int MT = WM * MB * 16;
  constexpr int PT = WN * NB * 16;
  constexpr int NIB = (PT * 4 + 255) / 256;  // B staging items (pixel, 16-byte quad) per thread
  constexpr int A_LANES = KT;                // threads along k when staging A
  constexpr int A_ROWS = 256 / A_LANES;      // rows per pass
  constexpr int NIA = (MT + A_ROWS - 1) / A_ROWS;

  __shared__ __attribute__((aligned(16))) unsigned char sA[2][MT * ROW_BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char sB[2][PT * ROW_BYTES];
  __shared__ __attribute__((aligned(16))) int2 ktab[2][KT];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int r = lane & 15, g = lane >> 4;

  const int tile_m = blockIdx.x % a.tiles_m;
  const int tile_p = blockIdx.x / a.tiles_m;
  const int o0 = tile_m * MT;
  const int p0 = tile_p * PT;
  const int split = blockIdx.z;
  const int kbeg = split * a.k_per_split;
  const int kend = min(a.K, kbeg + a.k_per_split);
  const int nslab = (kend - kbeg + KT - 1) / KT;

  const T* __restrict__ xg = (const T*)a.x;
  const T* __restrict__ wg = (const T*)a.w;

  // ---- per-thread staging state ----
  int b_base[NIB];
  unsigned b_mask[NIB];
  int b_row[NIB], b_quad[NIB];
#pragma unroll
  for (int j = 0; j < NIB; ++j) {
    int idx = t + 256 * j;
    int pi = idx % PT, q = idx / PT;
    const bool item = idx < PT * 4;
    b_row[j] = pi;
    b_quad[j] = item ? q : 0;
    unsigned pm = 0;
    int base = 0;
    int p = p0 + pi;
    if (item && p < a.P) {
      int n = p / a.HoWo;
      int rem = p - n * a.HoWo;
      int oy = rem / a.Wo;
      int ox = rem - oy * a.Wo;
      int iy0 = oy * a.stride - a.pad, ix0 = ox * a.stride - a.pad;
      base = (n * a.C * a.H + iy0) * a.W + ix0;
      for (int u = 0; u < a.KH; ++u)
        if ((unsigned)(iy0 + u) < (unsigned)a.H) pm |= 1u << u;
      for (int v = 0; v < a.KW; ++v)
        if ((unsigned)(ix0 + v) < (unsigned)a.W) pm |= 1u << (8 + v);
    }
    b_base[j] = base;
    b_mask[j] = pm;
  }
  const int a_k = t % A_LANES;
  const int a_row0 = t / A_LANES;

  auto write_table = [&](int slab, int slot) {
    if (t < KT) {
      int k = kbeg + slab * KT + t;
      int2 e;
      if (k < kend) {
        unsigned c = fast_div((unsigned)k, a.magic_khw);
        unsigned rr = (unsigned)k - c * (unsigned)a.KHW;
        unsigned u = fast_div(rr, a.magic_kw);
        unsigned v = rr - u * (unsigned)a.KW;
        e.x = (int)(c * (unsigned)a.HW + u * (unsigned)a.W + v);
        e.y = (int)((1u << u) | (1u << (8 + v)));
      } else {
        e.x = 0;
        e.y = (int)0x80000000u;  // never satisfied by a pixel mask
      }
      ktab[slot][t] = e;
    }
  };

  raw_t breg[NIB][EPI];
  raw_t areg[NIA];

  auto gload = [&](int slab, int slot) {
    const int k0 = kbeg + slab * KT;
    // A: weights, rows of KT contiguous k
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      int m = a_row0 + j * A_ROWS;
      int o = o0 + m;
      int k = k0 + a_k;
      raw_t v = 0;
      if (m < MT && o < a.O && k < kend)
        v = ((const raw_t*)wg)[(size_t)o * a.K + k];
      areg[j] = v;
    }
    // B: gathered input pixels
#pragma unroll
    for (int j = 0; j < NIB; ++j) {
      const int2* tab = &ktab[slot][b_quad[j] * EPI];
#pragma unroll
      for (int e = 0; e < EPI; ++e) {
        int2 ent = tab[e];
        raw_t v = 0;
        if ((b_mask[j] & (unsigned)ent.y) == (unsigned)ent.y)
          v = ((const raw_t*)xg)[b_base[j] + ent.x];
        breg[j][e] = v;
      }
    }
  };

  auto lds_store = [&](int buf) {
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      int m = a_row0 + j * A_ROWS;
      if (m < MT) *(raw_t*)&sA[buf][m * ROW_BYTES + a_k * (int)sizeof(T)] = areg[j];
    }
#pragma unroll
    for (int j = 0; j < NIB; ++j) {
      if (t + 256 * j < PT * 4) {
        uint4 pk;
        if constexpr (sizeof(T) == 4) {
          pk = make_uint4(breg[j][0], breg[j][1], breg[j][2], breg[j][3]);
        } else {
          pk = make_uint4((uint32_t)breg[j][0] | ((uint32_t)breg[j][1] << 16),
                          (uint32_t)breg[j][2] | ((uint32_t)breg[j][3] << 16),
                          (uint32_t)breg[j][4] | ((uint32_t)breg[j][5] << 16),
                          (uint32_t)breg[j][6] | ((uint32_t)breg[j][7] << 16));
        }
        *(uint4*)&sB[buf][b_row[j] * ROW_BYTES + b_quad[j] * 16] = pk;
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
  const int m_wave = o0 + wm * MB * 16;
  int mb_count = (a.O - m_wave + 15) / 16;
  mb_count = mb_count < 0 ? 0 : (mb_count > MB ? MB : mb_count);

  // ---- pipeline ----
  if (nslab > 0) {
    write_table(0, 0);
    __syncthreads();
    gload(0, 0);
    if (nslab > 1) write_table(1, 1);
    lds_store(0);
    __syncthreads();
  }
  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    if (s + 1 < nslab) gload(s + 1, (s + 1) & 1);
    if (s + 2 < nslab) write_table(s + 2, s & 1);

    uint4 bf[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
      bf[j] = *(const uint4*)&sB[buf][(wn * NB * 16 + j * 16 + r) * ROW_BYTES + g * 16];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      if (i < mb_count) {
        uint4 af = *(const uint4*)&sA[buf][(wm * MB * 16 + i * 16 + r) * ROW_BYTES + g * 16];
#pragma unroll
        for (int j = 0; j < NB; ++j) mma_frag<T>(af, bf[j], acc[i][j]);
      }
    }

    if (s + 1 < nslab) lds_store(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue ----
  // lane holds rows 4g..4g+3 (filters) of column r (pixel) of each block
  T* __restrict__ yg = (T*)a.y;
  const T* __restrict__ rg = (const T*)a.res;
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    int p = p0 + wn * NB * 16 + j * 16 + r;
    if (p >= a.P) continue;
    if (a.split_k > 1) {
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        if (i >= mb_count) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          int o = m_wave + i * 16 + 4 * g + v;
          if (o < a.O) a.partial[((size_t)split * a.O + o) * a.P + p] = acc[i][j][v];
        }
      }
    } else {
      int n = p / a.HoWo;
      int rem = p - n * a.HoWo;
      size_t pix = (size_t)n * a.O * a.HoWo + rem;
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        if (i >= mb_count) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          int o = m_wave + i * 16 + 4 * g + v;
          if (o < a.O) {
            float val = acc[i][j][v] + (a.bias ? a.bias[o] : 0.0f);
            size_t off = pix + (size_t)o * a.HoWo;
            if (rg) val += Elem<T>::to_f32(rg[off]);
            yg[off] = Elem<T>::from_f32(apply_act(val, a.act));
          }
        }
      }
    }
  }
}

// Sums the split-K partials in slice order (deterministic), then the epilogue.
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(ConvArgs a) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t total = (size_t)a.O * a.P;
  if (i >= total) return;
  int o = (int)(i / a.P);
  int p = (int)(i - (size_t)o * a.P);
  float s = 0.0f;
  for (int k = 0; k < a.split_k; ++k) s += a.partial[(size_t)k * total + i];
  s += a.bias ? a.bias[o] : 0.0f;
  int n = p / a.HoWo;
  int rem = p - n * a.HoWo;
  size_t off = ((size_t)n * a.O + o) * a.HoWo + rem;
  if (a.res) s += Elem<T>::to_f32(((const T*)a.res)[off]);
  ((T*)a.y)[off] = Elem<T>::from_f32(apply_act(s, a.act));
}

const TileVariant kTiles[] = {
    // wm wn mb nb
    {1, 4, 4, 4, 1},  // 64 x 256
    {1, 4, 8, 2, 1},  // 128 x 128
    {2, 2, 4, 4, 1},  // 128 x 128
    {1, 4, 2, 4, 1},  // 32 x 256
    {1, 4, 4, 2, 1},  // 64 x 128
    {1, 4, 1, 4, 1},  // 16 x 256
    {1, 4, 3, 4, 1},  // 48 x 256
    {1, 4, 2, 2, 1},  // 32 x 128
    {1, 4, 1, 2, 1},  // 16 x 128
    {1, 4, 4, 1, 1},  // 64 x 64
    {1, 4, 2, 1, 1},  // 32 x 64
    {1, 4, 8, 1, 1},  // 128 x 64
    {4, 1, 2, 7, 1},  // 128 x 112
    {2, 2, 4, 6, 1},  // 128 x 192
    {1, 4, 6, 3, 1},  // 96 x 192
    {1, 4, 1, 1, 1},  // 16 x 64
    {2, 2, 8, 4, 1},  // 256 x 128
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
const int kSplits[] = {1, 2, 4, 8, 16};
constexpr int kNumSplits = sizeof(kSplits) / sizeof(kSplits[0]);

template <typename T>
void launch_tile(int tile, dim3 grid, hipStream_t s, const ConvArgs& a) {
#define CASE(ID, WM_, WN_, MB_, NB_)                                                           \
  case ID:                                                                                     \
    hipLaunchKernelGGL((conv_igemm_kernel<T, WM_, WN_, MB_, NB_>), grid, dim3(256), 0, s, a);  \
    break;
  switch (tile) {
    CASE(0, 1, 4, 4, 4)
    CASE(1, 1, 4, 8, 2)
    CASE(2, 2, 2, 4, 4)
    CASE(3, 1, 4, 2, 4)
    CASE(4, 1, 4, 4, 2)
    CASE(5, 1, 4, 1, 4)
    CASE(6, 1, 4, 3, 4)
    CASE(7, 1, 4, 2, 2)
    CASE(8, 1, 4, 1, 2)
    CASE(9, 1, 4, 4, 1)
    CASE(10, 1, 4, 2, 1)
    CASE(11, 1, 4, 8, 1)
    CASE(12, 4, 1, 2, 7)
    CASE(13, 2, 2, 4, 6)
    CASE(14, 1, 4, 6, 3)
    CASE(15, 1, 4, 1, 1)
    CASE(16, 2, 2, 8, 4)
  }
#undef CASE
}

unsigned magic_for(unsigned d) {
  if (d <= 1) return 0;
  return (unsigned)((0x100000000ull + d - 1) / d);
}

int slab_k(int dt) { return dt == CPRUNE_F32 ? 16 : 32; }

}  // namespace

int num_variants() { return kNumTiles * kNumSplits; }

const TileVariant& variant(int id) {
  static TileVariant table[kNumTiles * kNumSplits];
  static bool init = false;
  if (!init) {
    for (int t = 0; t < kNumTiles; ++t)
      for (int s = 0; s < kNumSplits; ++s) {
        table[t * kNumSplits + s] = kTiles[t];
        table[t * kNumSplits + s].split_k = kSplits[s];
      }
    init = true;
  }
  return table[id];
}

bool variant_supports(const cprune_conv_desc& d, int v) {
  if (v < 0 || v >= num_variants()) return false;
  if (d.groups != 1) return false;
  const TileVariant& tv = variant(v);
  long K = (long)d.c_in * d.kh * d.kw;
  int kt = slab_k(d.dtype);
  long slabs = (K + kt - 1) / kt;
  if (tv.split_k > 1 && slabs < 2L * tv.split_k) return false;  // at least two slabs per slice
  return true;
}

size_t conv_ws_bytes(const cprune_conv_desc& d, int v) {
  if (d.groups != 1) return 0;
  int ho = conv_out_dim(d.h, d.kh, d.stride, d.pad), wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  size_t op = (size_t)d.c_out * d.n * ho * wo * sizeof(float);
  if (v >= 0) {
    int sk = variant(v).split_k;
    return sk > 1 ? op * sk : 0;
  }
  size_t best = 0;
  for (int i = 0; i < num_variants(); ++i)
    if (variant_supports(d, i)) {
      size_t b = conv_ws_bytes(d, i);
      if (b > best) best = b;
    }
  return best;
}

int launch_conv_dense(const cprune_conv_desc& d, const void* x, const void* w, const float* bias,
                      const void* residual, void* y, int v, void* ws, hipStream_t s) {
  const TileVariant& tv = variant(v);
  ConvArgs a;
  a.x = x; a.w = w; a.bias = bias; a.res = residual; a.y = y; a.partial = (float*)ws;
  a.N = d.n; a.C = d.c_in; a.H = d.h; a.W = d.w; a.O = d.c_out; a.KH = d.kh; a.KW = d.kw;
  a.stride = d.stride; a.pad = d.pad;
  a.Ho = conv_out_dim(d.h, d.kh, d.stride, d.pad);
  a.Wo = conv_out_dim(d.w, d.kw, d.stride, d.pad);
  a.K = d.c_in * d.kh * d.kw;
  a.HoWo = a.Ho * a.Wo;
  a.P = d.n * a.HoWo;
  a.HW = d.h * d.w;
  a.KHW = d.kh * d.kw;
  a.magic_khw = magic_for((unsigned)a.KHW);
  a.magic_kw = magic_for((unsigned)a.KW);
  a.act = d.act;
  const int mt = tv.tile_m(), pt = tv.tile_p();
  a.tiles_m = (a.O + mt - 1) / mt;
  const int tiles_p = (a.P + pt - 1) / pt;
  const int kt = slab_k(d.dtype);
  const int slabs = (a.K + kt - 1) / kt;
  a.split_k = tv.split_k;
  a.k_per_split = ((slabs + tv.split_k - 1) / tv.split_k) * kt;
  dim3 grid((unsigned)(a.tiles_m * tiles_p), 1, (unsigned)a.split_k);
  const int tile = v / kNumSplits;
  if (d.dtype == CPRUNE_F32) launch_tile<float>(tile, grid, s, a);
  else if (d.dtype == CPRUNE_F16) launch_tile<_Float16>(tile, grid, s, a);
  else launch_tile<__bf16>(tile, grid, s, a);
  CPRUNE_LAUNCH_CHECK();
  if (a.split_k > 1) {
    size_t total = (size_t)a.O * a.P;
    dim3 g2((unsigned)((total + 255) / 256));
    if (d.dtype == CPRUNE_F32) hipLaunchKernelGGL(splitk_reduce_kernel<float>, g2, dim3(256), 0, s, a);
    else if (d.dtype == CPRUNE_F16) hipLaunchKernelGGL(splitk_reduce_kernel<_Float16>, g2, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(splitk_reduce_kernel<__bf16>, g2, dim3(256), 0, s, a);
    CPRUNE_LAUNCH_CHECK();
  }
  return CPRUNE_OK;
}

}  // namespace cprune
