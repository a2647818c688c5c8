// Dense layer whose reduction is one contiguous run of memory per output pixel (a 1x1 /
// stride 1 convolution, a fully connected layer, a 2x2 map run as one matrix), channels-last,
// for the case of FEW pixels and a LONG reduction: the late layers of a network on small
// inputs.  There the other kernels either leave most compute units idle (one work-group per
// output tile) or cut the reduction between work-groups and need a second launch to add the
// pieces up.  Here a work-group owns 16 filters x 16 * NB pixels and its KW wavefronts split
// the reduction between them: each multiplies its share straight from global memory (both
// operands are k-contiguous, so a lane's MFMA operand is one 16-byte load; nothing is staged
// because no two wavefronts of the group read the same bytes), then the partial sums meet in
// LDS and the first NB wavefronts run the epilogue.  One launch, no scratch buffer.
//
// Same MFMA blocks, lane layout and k-permutation as the other dense kernels.
#pragma once
#include "conv_patch_kernel.hpp"

namespace cprune {

template <typename T, int NB, int KW>
__global__ __launch_bounds__(64 * KW) void conv_ksplit_kernel(ConvArgs a) {
  constexpr int ES = (int)sizeof(T);
  constexpr int U = 4;                          // 64-byte rounds per batch of loads
  constexpr int NS = NB >= 4 ? 1 : 4 / NB;      // accumulator sets (see mma_round)
  static_assert(KW * NB <= 32, "partial sums fit LDS");

  __shared__ float4_t red[KW][NB][64];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // uniform: it decides scalar load offsets
  const int r = lane & 15, g4 = lane >> 4;

  // each XCD (own L2) takes a contiguous stretch of the tile order; pixel tiles run fastest,
  // so the groups of a stretch share their filter rows
  int g;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    g = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  const int tile_m = (int)fast_div((unsigned)g, a.magic_tp), tile_p = g - tile_m * a.tiles_p;
  const int o0 = tile_m * 16, p0 = tile_p * (16 * NB);

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t wr = make_rsrc(a.w, a.w_bytes);
  // requested now, used in the epilogue: on a short layer a load issued there would be waited for in full
  const float4_t bias4 = load_bias4(a.bias, a.O, o0 + 4 * g4);
  const unsigned row_bytes = (unsigned)a.K * ES;          // a multiple of 16: channel strides are whole vectors
  const int rounds = (int)((row_bytes + 63) / 64);
  const int lo = (int)((long)wave * rounds / KW), hi = (int)((long)(wave + 1) * rounds / KW);

  // weights: rows of the reduction, or (w_packed) the fragment-ordered copy, where one wavefront-wide load is
  // 1 KiB of consecutive memory instead of 16 half cache lines
  const unsigned a_off = a.w_packed ? (unsigned)lane * 16u
                                    : ((o0 + r < a.O) ? (unsigned)(o0 + r) * row_bytes + g4 * 16 : kOutOfRange);
  const unsigned a_tile = a.w_packed ? (unsigned)(tile_m * rounds) * 1024u : 0u;
  const unsigned a_step = a.w_packed ? 1024u : 64u;
  unsigned b_off[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int p = p0 + j * 16 + r;
    b_off[j] = p < a.P ? (unsigned)p * row_bytes + g4 * 16 : kOutOfRange;
  }

  float4_t accs[NS][1][NB];
#pragma unroll
  for (int q = 0; q < NS; ++q)
#pragma unroll
    for (int j = 0; j < NB; ++j) accs[q][0][j] = (float4_t){0.f, 0.f, 0.f, 0.f};

  // two register sets of U rounds each: one is multiplied while the other is in flight
  uint4 af0[U][1], bf0[U][NB], af1[U][1], bf1[U][NB];
  auto gload = [&](int r0, uint4 (&fa)[U][1], uint4 (&fb)[U][NB]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int rnd = r0 + u;
      const unsigned inval = (unsigned)(rnd >= hi || (unsigned)rnd * 64 + g4 * 16 >= row_bytes) << 31;
      fa[u][0] = load_b128(wr, a_off | inval, a_tile + (unsigned)rnd * a_step);
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[u][j] = load_b128(xr, b_off[j] | inval, (unsigned)rnd * 64);
    }
  };
  auto multiply = [&](const uint4 (&fa)[U][1], const uint4 (&fb)[U][NB]) {
#pragma unroll
    for (int u = 0; u < U; ++u) mma_round<T, 1, NB, 1, NS>(fa[u], fb[u], accs, u);
  };
  if (lo < hi) gload(lo, af0, bf0);
  for (int r0 = lo; r0 < hi; r0 += 2 * U) {
    const bool second = r0 + U < hi;
    if (second) gload(r0 + U, af1, bf1);
    multiply(af0, bf0);
    if (r0 + 2 * U < hi) gload(r0 + 2 * U, af0, bf0);
    if (second) multiply(af1, bf1);
  }

#pragma unroll
  for (int j = 0; j < NB; ++j) {
    float4_t s = accs[0][0][j];
#pragma unroll
    for (int q = 1; q < NS; ++q) s += accs[q][0][j];
    red[wave][j][lane] = s;
  }
  __syncthreads();
  if (wave >= NB) return;

  // wavefront j adds up pixel block j and stores it
  float4_t acc = red[0][wave][lane];
#pragma unroll
  for (int w = 1; w < KW; ++w) acc += red[w][wave][lane];
  const int p = p0 + wave * 16 + r;
  if (p >= a.P) return;
  nhwc_store4<T>(a, acc, p, o0 + 4 * g4, bias4);
}

// Variants: id, nb (16-pixel blocks per work-group), kw (wavefronts splitting the reduction)
#define CPRUNE_KSPLIT_LIST(X) \
  X(0, 1, 4)                  \
  X(1, 1, 8)                  \
  X(2, 1, 16)                 \
  X(3, 2, 4)                  \
  X(4, 2, 8)                  \
  X(5, 4, 4)                  \
  X(6, 4, 8)                  \
  X(7, 1, 2)                  \
  X(8, 2, 2)

constexpr int kNumKsplit = 9;

template <typename T>
inline void launch_ksplit(int id, dim3 grid, hipStream_t s, const ConvArgs& a) {
#define CPRUNE_KSPLIT_CASE(ID, NB_, KW_)                                                          \
  case ID:                                                                                        \
    hipLaunchKernelGGL((conv_ksplit_kernel<T, NB_, KW_>), grid, dim3(64 * KW_), 0, s, a);         \
    break;
  switch (id) { CPRUNE_KSPLIT_LIST(CPRUNE_KSPLIT_CASE) }
#undef CPRUNE_KSPLIT_CASE
}

void launch_conv_ksplit_f32(int id, dim3 grid, hipStream_t s, const ConvArgs& a);
void launch_conv_ksplit_f16(int id, dim3 grid, hipStream_t s, const ConvArgs& a);
void launch_conv_ksplit_bf16(int id, dim3 grid, hipStream_t s, const ConvArgs& a);

}  // namespace cprune
