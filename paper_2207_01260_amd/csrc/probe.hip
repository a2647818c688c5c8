// Measured ceilings of the device, next to which kernel throughput is reported: the
// rate of back-to-back MFMA instructions on register operands (no memory traffic at all),
// and the rate of a plain device-to-device copy.
#include "common.hpp"
#include <functional>

namespace cprune {
namespace {

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kProbeGroups = 2048;   // 8 work-groups of 4 wavefronts per compute unit

// DT 0: fp32, 1: fp16, 2: bf16.  BIG 0: 16x16 blocks (x4 fp32, x32 16-bit), 16 independent
// accumulators; BIG 1: 32x32 blocks (x2 fp32, x16 16-bit), 4 accumulators.
template <int DT, int BIG>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* out, int iters, float seed) {
  const float av = seed + (float)threadIdx.x * 1e-3f, bv = seed * 0.5f;
  half8_t ah, bh;
  bf16x8_t ab, bb;
#pragma unroll
  for (int e = 0; e < 8; ++e) { ah[e] = (_Float16)av; bh[e] = (_Float16)bv; ab[e] = (__bf16)av; bb[e] = (__bf16)bv; }
  float s = 0.f;
  if constexpr (BIG == 0) {
    constexpr int NA = 16;
    float4_t acc[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) acc[i] = (float4_t){0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < NA; ++i) {
        if constexpr (DT == 0) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[i], 0, 0, 0);
        else if constexpr (DT == 1) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bh, acc[i], 0, 0, 0);
        else acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, bb, acc[i], 0, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < NA; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  } else {
    constexpr int NA = 4;
    float16_t acc[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < NA; ++i) {
        if constexpr (DT == 0) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i], 0, 0, 0);
        else if constexpr (DT == 1) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, acc[i], 0, 0, 0);
        else acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bb, acc[i], 0, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) s += acc[i][j];
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Streaming probes: MODE 0 copies, 1 only reads (xor of everything read kept alive by a never-true store), 2 only
// writes.  A thread moves U pieces of 16 bytes per step, all U loads issued before the first store; NT: loads and
// stores marked non-temporal (streamed past the caches).  Grid-stride over steps of U * 256 pieces per work-group.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <int MODE, int U, bool NT>
__global__ __launch_bounds__(256) void stream_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                           size_t n16) {
  const size_t per_step = (size_t)U * 256;
  uint4 acc = {0u, 0u, 0u, 0u};
  for (size_t base = (size_t)blockIdx.x * per_step; base < n16; base += (size_t)gridDim.x * per_step) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t i = base + (size_t)u * 256 + threadIdx.x;
      if (MODE == 2) v[u] = uint4{(unsigned)i, 1u, 2u, 3u};
      else if (i < n16) v[u] = NT ? __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src) + i)) : src[i];
      else v[u] = uint4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t i = base + (size_t)u * 256 + threadIdx.x;
      if (MODE == 1) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
      else if (i < n16) {
        if (NT) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v[u]), reinterpret_cast<u32x4*>(dst) + i);
        else dst[i] = v[u];
      }
    }
  }
  if (MODE == 1 && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u && n16 == 1) dst[0] = acc;   // keeps the loads alive
}

// Reads of L2-resident data by 16-byte-per-lane buffer loads, as the kernels that take MFMA operands straight
// from global memory issue them.  Every work-group (4 wavefronts) walks `passes` times over a region of
// 16 rows x row_bytes (larger than the vector cache); 16 work-groups share a region, as the work-groups of
// one filter tile do.  PAT 0: a wavefront-wide load covers 1 KiB of consecutive memory (8 whole cache
// lines).  PAT 1: 16 rows x 64 bytes (16 half lines), the shape of an operand tile in a row-major matrix.
template <int PAT>
__global__ __launch_bounds__(256) void l2_probe_kernel(const char* base, unsigned row_bytes, int regions, int passes,
                                                       float* out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned region = 16u * row_bytes;
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(base) + (size_t)(blockIdx.x % regions) * region, 0, (int)region, 0x00020000);
  const unsigned steps = region / 1024 / 4;   // loads per wavefront and pass (a ragged rest is not read)
  const unsigned cols = row_bytes / 64;
  uint4 acc = {0u, 0u, 0u, 0u};
  for (int p = 0; p < passes; ++p) {
    for (unsigned i = 0; i + 4 <= steps; i += 4) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const unsigned step = (i + u) * 4 + wave;
        unsigned off;
        if (PAT == 0) off = step * 1024 + lane * 16;
        else off = (unsigned)(lane & 15) * row_bytes + (step % cols) * 64 + (lane >> 4) * 16;
        v[u] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) out[0] = 1.f;   // keeps the loads alive
}

int timed(hipStream_t s, int reps, float* ms_out, const std::function<void()>& launch) {
  hipEvent_t e0, e1;
  CPRUNE_HIP_TRY(hipEventCreate(&e0));
  hipError_t e = hipEventCreate(&e1);
  if (e != hipSuccess) { hipEventDestroy(e0); set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
  float best = 0.f;
  launch();   // warm-up
  for (int r = 0; r < reps && e == hipSuccess; ++r) {
    e = hipEventRecord(e0, s);
    launch();
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (r == 0 || ms < best) best = ms;
  }
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  if (e != hipSuccess) { set_last_hip_error(e); return CPRUNE_ERR_DEVICE; }
  *ms_out = best;
  return CPRUNE_OK;
}

}  // namespace
}  // namespace cprune

using namespace cprune;

extern "C" size_t cprune_probe_scratch_bytes(void) { return (size_t)kProbeGroups * 256 * sizeof(float); }

extern "C" int cprune_probe_mfma(cprune_dtype dtype, void* scratch, size_t scratch_bytes, float* tflops_out,
                                 void* stream) {
  if (!scratch || !tflops_out || !dtype_ok(dtype)) return CPRUNE_ERR_INVALID_ARG;
  if (scratch_bytes < cprune_probe_scratch_bytes()) return CPRUNE_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int iters = 2000;
  float best = 0.f;
  for (int big = 0; big < 2; ++big) {
    float ms = 0.f;
    int rc = timed(s, 3, &ms, [&]() {
#define CPRUNE_PROBE(DT, BIG) hipLaunchKernelGGL((mfma_probe_kernel<DT, BIG>), dim3(kProbeGroups), dim3(256), 0, s, (float*)scratch, iters, 1.0f)
      if (dtype == CPRUNE_F32) { if (big) CPRUNE_PROBE(0, 1); else CPRUNE_PROBE(0, 0); }
      else if (dtype == CPRUNE_F16) { if (big) CPRUNE_PROBE(1, 1); else CPRUNE_PROBE(1, 0); }
      else { if (big) CPRUNE_PROBE(2, 1); else CPRUNE_PROBE(2, 0); }
#undef CPRUNE_PROBE
    });
    if (rc != CPRUNE_OK) return rc;
    // 16x16x4 and 32x32x2 (fp32) are 2048 / 4096 FLOP, 16x16x32 and 32x32x16 (16-bit) 16384 / 32768
    const double flop_per_mfma = (dtype == CPRUNE_F32 ? 2048.0 : 16384.0) * (big ? 2.0 : 1.0);
    const double flops = (double)kProbeGroups * 4 * iters * (big ? 4 : 16) * flop_per_mfma;
    const float t = (float)(flops / (ms * 1e-3) / 1e12);
    if (t > best) best = t;
  }
  *tflops_out = best;
  return CPRUNE_OK;
}

// The fastest of several launch shapes of one streaming mode: pieces per thread 4 or 8, cached or non-temporal
// accesses, one step per work-group or 8 / 16 resident work-groups per compute unit walking the buffer.
template <int MODE>
static int probe_stream(const void* src, void* dst, size_t bytes, float* ms_out, hipStream_t s) {
  const size_t n16 = bytes / 16;
  float best = 0.f;
  bool have = false;
  for (int shape = 0; shape < 8; ++shape) {
    const int u = (shape & 1) ? 8 : 4;
    const bool nt = (shape & 2) != 0;
    const size_t cover = (n16 + (size_t)u * 256 - 1) / ((size_t)u * 256);
    size_t groups = (shape & 4) ? (size_t)256 * 16 : cover;
    if (groups > cover) groups = cover;
    if (groups > 0x7fffffffu) continue;
    float ms = 0.f;
    int rc = timed(s, 4, &ms, [&]() {
#define CPRUNE_STREAM(U, NT) hipLaunchKernelGGL((stream_probe_kernel<MODE, U, NT>), dim3((unsigned)groups), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n16)
      if (u == 4) { if (nt) CPRUNE_STREAM(4, true); else CPRUNE_STREAM(4, false); }
      else { if (nt) CPRUNE_STREAM(8, true); else CPRUNE_STREAM(8, false); }
#undef CPRUNE_STREAM
    });
    if (rc != CPRUNE_OK) return rc;
    if (!have || ms < best) { best = ms; have = true; }
  }
  *ms_out = best;
  return CPRUNE_OK;
}

extern "C" int cprune_probe_copy(const void* src, void* dst, size_t bytes, float* gbps_out, void* stream) {
  if (!src || !dst || !gbps_out || bytes < 16 || (bytes & 15)) return CPRUNE_ERR_INVALID_ARG;
  float ms = 0.f;
  int rc = probe_stream<0>(src, dst, bytes, &ms, (hipStream_t)stream);
  if (rc != CPRUNE_OK) return rc;
  *gbps_out = (float)(2.0 * (double)bytes / (ms * 1e-3) / 1e9);   // bytes read + bytes written
  return CPRUNE_OK;
}

extern "C" int cprune_probe_read(const void* src, void* scratch16, size_t bytes, float* gbps_out, void* stream) {
  if (!src || !scratch16 || !gbps_out || bytes < 32 || (bytes & 15)) return CPRUNE_ERR_INVALID_ARG;
  float ms = 0.f;
  int rc = probe_stream<1>(src, scratch16, bytes, &ms, (hipStream_t)stream);
  if (rc != CPRUNE_OK) return rc;
  *gbps_out = (float)((double)bytes / (ms * 1e-3) / 1e9);
  return CPRUNE_OK;
}

extern "C" int cprune_probe_write(void* dst, size_t bytes, float* gbps_out, void* stream) {
  if (!dst || !gbps_out || bytes < 16 || (bytes & 15)) return CPRUNE_ERR_INVALID_ARG;
  float ms = 0.f;
  int rc = probe_stream<2>(dst, dst, bytes, &ms, (hipStream_t)stream);
  if (rc != CPRUNE_OK) return rc;
  *gbps_out = (float)((double)bytes / (ms * 1e-3) / 1e9);
  return CPRUNE_OK;
}

extern "C" size_t cprune_probe_l2_bytes(void) { return (size_t)16 * 16 * 10944; }   // 16 regions of 16 rows

extern "C" int cprune_probe_l2_read(int pattern, const void* buf, size_t buf_bytes, float* scratch,
                                    float* gbps_per_cu_out, void* stream) {
  if (!buf || !scratch || !gbps_per_cu_out || (pattern != 0 && pattern != 1)) return CPRUNE_ERR_INVALID_ARG;
  if (buf_bytes < cprune_probe_l2_bytes()) return CPRUNE_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  int dev = 0, cus = 0;
  CPRUNE_HIP_TRY(hipGetDevice(&dev));
  CPRUNE_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const unsigned row_bytes = 10944;   // 171 columns of 64 bytes: the filter row of a 304-channel 3x3 layer
  const int passes = 20;
  float ms = 0.f;
  int rc = timed(s, 3, &ms, [&]() {
    if (pattern == 0) hipLaunchKernelGGL(l2_probe_kernel<0>, dim3((unsigned)cus), dim3(256), 0, s, (const char*)buf, row_bytes, 16, passes, scratch);
    else hipLaunchKernelGGL(l2_probe_kernel<1>, dim3((unsigned)cus), dim3(256), 0, s, (const char*)buf, row_bytes, 16, passes, scratch);
  });
  if (rc != CPRUNE_OK) return rc;
  // bytes one work-group (= one compute unit: the grid has one group per unit) reads
  const double steps = (double)((16u * row_bytes / 1024 / 4) / 4 * 4);
  const double bytes = steps * 4 * 1024 * passes;
  *gbps_per_cu_out = (float)(bytes / (ms * 1e-3) / 1e9);
  return CPRUNE_OK;
}
