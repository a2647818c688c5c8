// 3x3 / stride 1 / pad 1 dense layer, channels-last, for SMALL maps with MANY channels (the late
// layers of a network on small inputs: a few hundred 16 x 16 output blocks, reductions of a few
// thousand).  The tiled kernels give such a layer about one work-group of four wavefronts per
// compute unit, which march in step between barriers: staging, fragment reads and MFMAs of a unit
// then run one after the other and the matrix pipe idles half the time; and a grid of slightly
// more groups than units runs two rounds.
//
// Here a wavefront shares nothing with its neighbours until the very end.  A work-group owns 16
// filters x NP * NB output blocks (a block = one 4 x 4 pixel tile of one image) and cuts the
// reduction into KS slices at (channel chunk, tap) granularity: NP * KS wavefronts, each multiplying
// NB blocks over one slice.  A wavefront stages the 6 x 6 input patches of its blocks in LDS of its
// own (taps are shifted reads of them; no barrier: the LDS serves one wavefront's accesses in
// order) and takes its weight fragments straight from global memory, where they lie packed in the order the
// lanes want them (one 16-byte load per lane and tap, 1 KiB of consecutive memory per wavefront: half
// lines cost the vector cache twice the time; used for all NB blocks).  With NP = 1 no byte is fetched twice by a
// group; with NP > 1 the wavefronts of a slice read the same weights through the vector cache.
// Every SIMD holds wavefronts at different points of their chunks, so one's loads and LDS
// traffic hide behind another's MFMAs.  The slices meet in LDS at the end (the only two
// barriers) and wavefront j stores block j.  NP * NB also chooses how evenly a layer's blocks
// spread over the compute units (5 turns 304 four-block tiles into 247 five-block ones).
// With a batch of one image a layer is a handful of blocks: then one block per group and 4 to 16
// slices of the reduction (NP = NB = 1) put the most wavefronts on it, and that is what wins there.
//
// Same MFMA blocks, lane layout and k-permutation as the other dense kernels.
#pragma once
#include <atomic>
#include "conv_patch_kernel.hpp"

namespace cprune {

template <typename T, int NP, int NB, int KS>
__global__ __launch_bounds__(64 * NP * KS) void conv_wave_kernel(PatchArgs a) {
  constexpr int ES = (int)sizeof(T);
  constexpr int EPI = 16 / ES;            // elements per quad
  constexpr int CC = 4 * EPI;             // channels per chunk: one 64-byte round per tap
  constexpr int NW = NP * KS;
  constexpr int NBLK = NP * NB;           // blocks per group
  constexpr int PW = 6, NPATCH = 36;      // input patch of a 4 x 4 output tile
  constexpr int BROW = 64 + 16;           // patch pixel: the chunk's channels + 16 pad
  constexpr int PBUF = NPATCH * BROW;
  constexpr int NIB = (NPATCH * 4 + 63) / 64;
  constexpr int NS = NB >= 4 ? 1 : 4 / NB;   // accumulator sets (see mma_round)
  static_assert(NW <= 16, "at most 1024 threads");

  // dynamic LDS: [NW][NB][PBUF] patches; at the end the same bytes hold [NW][NB][64] partial sums
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // uniform: blocks and slice are scalar
  const int pw = wave % NP, kg = wave / NP;
  const int r = lane & 15, g4 = lane >> 4;

  // group decode; each XCD (own L2) gets one contiguous stretch of the group order
  int grp;
  {
    const int G = gridDim.x;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int q = G >> 3, rem = G & 7;
    grp = xcd * q + (xcd < rem ? xcd : rem) + local;
  }
  // a.tiles_n: groups along the block list (blocks = images x tiles_y x tiles_x, NBLK per group)
  const int q_s = (int)fast_div((unsigned)grp, a.magic_s), q_m = (int)fast_div((unsigned)grp, a.magic_m);
  const int tile_m = a.m_major ? q_s : grp - q_m * a.tiles_m;
  const int gp = a.m_major ? grp - q_s * a.tiles_n : q_m;
  const int o0 = tile_m * 16;
  const int blocks = a.N * a.tiles_y * a.tiles_x;
  const int txy = a.tiles_x * a.tiles_y;
  const int u0 = gp * NBLK + pw * NB;     // first block of this wavefront
  const bool any = u0 < blocks;

  const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t wr = make_rsrc(a.w, a.w_bytes);
  // requested now, used in the epilogue: on a short layer a load issued there would be waited for in full
  const float4_t bias4 = load_bias4(a.bias, a.O, o0 + 4 * g4);

  // ---- staging items of the patches: (block, patch pixel, quad) ----
  unsigned b_off[NB][NIB];
  int b_lds[NIB];
#pragma unroll
  for (int i = 0; i < NIB; ++i) {
    const int idx = lane + 64 * i;
    const int q = idx & 3, pp = idx >> 2;
    const bool item = pp < NPATCH;
    const int py = pp / PW, px = pp - py * PW;
    b_lds[i] = item ? pp * BROW + q * 16 : PBUF - 16;   // no item: the last row's pad, which nobody reads
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int u = u0 + j;
      const int n = (int)fast_div((unsigned)u, a.magic_xy), rest = u - n * txy;
      const int by = (int)fast_div((unsigned)rest, a.magic_x);
      const int iy = by * 4 + py - 1, ix = (rest - by * a.tiles_x) * 4 + px - 1;
      const bool inside = item && u < blocks && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
      b_off[j][i] = inside ? (unsigned)(((n * a.H + iy) * a.W + ix) * a.Cp + q * EPI) * ES : kOutOfRange;
    }
  }
  // weights come packed in fragment order, [filter tile][chunk][tap][lane][16 bytes] (zeros past the last
  // filter and channel): the wavefront's operand of one tap is 1 KiB of consecutive memory
  const unsigned a_off = any ? (unsigned)lane * 16u : kOutOfRange;
  // the lane's pixel of the 4 x 4 tile inside the patch (tap (0,0) corner)
  const int b_frag = ((r >> 2) * PW + (r & 3)) * BROW + g4 * 16;

  unsigned char* const myB = smem + wave * (NB * PBUF);

  // the slice of this wavefront, in (chunk, tap) units
  const int nchunk = (a.Cp + CC - 1) / CC;
  const int units = nchunk * 9;
  const int ulo = (int)((long)kg * units / KS), uhi = (int)((long)(kg + 1) * units / KS);
  const int clo = ulo / 9, chi = (uhi + 8) / 9;

  uint4 breg[NB][NIB], a0[9], a1[9];
  auto load_patch = [&](int c) {
    const int c0 = c * CC;
#pragma unroll
    for (int i = 0; i < NIB; ++i) {
      const unsigned inval = (unsigned)(c0 + ((lane + 64 * i) & 3) * EPI >= a.Cp) << 31;
#pragma unroll
      for (int j = 0; j < NB; ++j) breg[j][i] = load_b128(xr, b_off[j][i] | inval, (unsigned)(c0 * ES));
    }
  };
  auto store_patch = [&]() {
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int i = 0; i < NIB; ++i) *(uint4*)&myB[j * PBUF + b_lds[i]] = breg[j][i];
  };
  // taps outside the slice are flagged out of range: zeros, no memory traffic (their MFMAs are skipped)
  auto load_weights = [&](int c, uint4 (&fa)[9]) {
    const unsigned base = (unsigned)((tile_m * nchunk + c) * 9) * 1024u;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int u = c * 9 + tap;
      const unsigned inval = (unsigned)(u < ulo || u >= uhi) << 31;
      fa[tap] = load_b128(wr, a_off | inval, base + (unsigned)tap * 1024u);
    }
  };

  float4_t accs[NS][1][NB];
#pragma unroll
  for (int q = 0; q < NS; ++q)
#pragma unroll
    for (int j = 0; j < NB; ++j) accs[q][0][j] = (float4_t){0.f, 0.f, 0.f, 0.f};

  // One chunk: its patches (loaded a chunk ago) go to LDS, then the loads of the next chunk (patches
  // and the other weight set) are issued, then the taps of the slice.  Every load in flight at the top
  // of a chunk is one the chunk needs, so the wait there is exact: the compiler cannot count loads in
  // flight across the loop's back edge and, asked to wait for the older of two batches, waits for both.
  auto chunk = [&](int c, uint4 (&fa)[9], uint4 (&fn)[9]) {
    store_patch();
    if (c + 1 < chi) {
      load_patch(c + 1);
      load_weights(c + 1, fn);
    }
    uint4 af[1], bf[2][NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) bf[0][j] = *(const uint4*)&myB[j * PBUF + b_frag];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      if (tap + 1 < 9) {
        const int nt = tap + 1;
#pragma unroll
        for (int j = 0; j < NB; ++j)
          bf[nt & 1][j] = *(const uint4*)&myB[j * PBUF + b_frag + ((nt / 3) * PW + (nt % 3)) * BROW];
      }
      const int u = c * 9 + tap;
      if (u >= ulo && u < uhi) {
        af[0] = fa[tap];
        mma_round<T, 1, NB, 1, NS>(af, bf[tap & 1], accs, tap);
      }
    }
  };

  if (any && clo < chi) {
    load_patch(clo);
    load_weights(clo, a0);
    for (int c = clo; c < chi; c += 2) {
      chunk(c, a0, a1);
      if (c + 1 < chi) chunk(c + 1, a1, a0);
    }
  }

  // ---- the slices meet: every wavefront leaves its sums where its patches were ----
  __syncthreads();              // (every wavefront gets here) all patch reads are done
  float4_t* const red = (float4_t*)smem;    // [kg][block of the group][lane]
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    float4_t sacc = accs[0][0][j];
#pragma unroll
    for (int q = 1; q < NS; ++q) sacc += accs[q][0][j];
    red[((size_t)kg * NBLK + pw * NB + j) * 64 + lane] = sacc;
  }
  __syncthreads();

  // ---- epilogue: wavefront b adds up block b; lane holds filters o0 + 4 * g4 .. + 3 of pixel r ----
  ConvArgs e;
  e.bias = a.bias; e.res = a.res; e.y = a.y; e.O = a.O; e.Cop = a.Cop; e.act = a.act; e.vec_out = a.vec_out; e.pool4 = 0;
  const int ty = r >> 2, tx = r & 3;
  const int o = o0 + 4 * g4;
  for (int b = wave; b < NBLK; b += NW) {
    const int u = gp * NBLK + b;
    if (u >= blocks) break;
    float4_t acc = red[(size_t)b * 64 + lane];
#pragma unroll
    for (int k = 1; k < KS; ++k) acc += red[((size_t)k * NBLK + b) * 64 + lane];
    const int n = (int)fast_div((unsigned)u, a.magic_xy), rest = u - n * txy;
    const int by = (int)fast_div((unsigned)rest, a.magic_x);
    const int oy = by * 4 + ty, ox = (rest - by * a.tiles_x) * 4 + tx;
    if (!a.pool) {
      if (oy < a.H && ox < a.W) nhwc_store4<T>(e, acc, (n * a.H + oy) * a.W + ox, o, bias4);
    } else {
      // bias + activation, then the max over each 2x2 window (partners: lanes r ^ 1 and r ^ 4); the
      // activation is monotone, so max(act(.)) equals act-then-pool.  The even/even corner stores.
      ConvArgs ep = e;
      ep.act = CPRUNE_ACT_NONE;
      ep.bias = nullptr;
      float4_t m;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float x = apply_act(acc[c] + bias4[c], a.act);
        x = fmaxf(x, __shfl_xor(x, 1, 64));
        x = fmaxf(x, __shfl_xor(x, 4, 64));
        m[c] = x;
      }
      if (!((ty | tx) & 1) && oy < a.H && ox < a.W)
        nhwc_store4<T>(ep, m, (n * (a.H >> 1) + (oy >> 1)) * (a.W >> 1) + (ox >> 1), o, (float4_t){0.f, 0.f, 0.f, 0.f});
    }
  }
}

// Variants: id, np (wavefronts along the blocks), nb (4 x 4 output blocks per wavefront), ks (slices
// of the reduction); np * ks wavefronts, np * nb blocks per work-group
#define CPRUNE_WAVE_LIST(X) \
  X(0, 1, 4, 4) \
  X(1, 1, 5, 4) \
  X(2, 1, 5, 8) \
  X(3, 2, 3, 2) \
  X(4, 5, 1, 3) \
  X(5, 5, 1, 2) \
  X(6, 4, 1, 4) \
  X(7, 2, 2, 4) \
  X(8, 2, 3, 4) \
  X(9, 2, 2, 2) \
  X(10, 4, 1, 2) \
  X(11, 3, 2, 4) \
  X(12, 1, 1, 16) \
  X(13, 1, 1, 8) \
  X(14, 1, 2, 8) \
  X(15, 2, 1, 8) \
  X(16, 1, 1, 4) \
  X(17, 1, 2, 4)

constexpr int kNumWave = 18;

constexpr size_t wave_lds_bytes(int np, int nb, int ks) { return (size_t)np * ks * nb * (36 * 80); }

template <typename T>
inline int launch_wave(int id, dim3 grid, hipStream_t s, const PatchArgs& a) {
#define CPRUNE_WAVE_CASE(ID, NP_, NB_, KS_)                                                                \
  case ID: {                                                                                               \
    constexpr size_t lds = wave_lds_bytes(NP_, NB_, KS_);                                                  \
    static_assert(lds <= 160 * 1024, "patches (the sums at the end need less)");                           \
    static std::atomic<bool> raised{false};   /* more than the default 64 KiB of LDS has to be asked for once */ \
    if (lds > 65536 && !raised.load(std::memory_order_relaxed)) {                                             \
      CPRUNE_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_wave_kernel<T, NP_, NB_, KS_>), \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));           \
      raised.store(true, std::memory_order_relaxed);                                                          \
    }                                                                                                      \
    hipLaunchKernelGGL((conv_wave_kernel<T, NP_, NB_, KS_>), grid, dim3(64 * NP_ * KS_), lds, s, a);       \
    break;                                                                                                 \
  }
  switch (id) { CPRUNE_WAVE_LIST(CPRUNE_WAVE_CASE) default: return CPRUNE_ERR_UNSUPPORTED; }
#undef CPRUNE_WAVE_CASE
  return CPRUNE_OK;
}

int launch_conv_wave_f32(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
int launch_conv_wave_f16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);
int launch_conv_wave_bf16(int id, dim3 grid, hipStream_t s, const PatchArgs& a);

}  // namespace cprune
