// Measurement aids: what this chip actually sustains on the two resources the roofline figures are quoted
// against.  Neither is part of the method; bench.py times them next to the real kernels so that every report
// can state a fraction of the datasheet peak and a fraction of the measured ceiling.
#include "ltea_common.h"
#include "../../include/ltea.h"

namespace ltea {
namespace {

constexpr int kDiagThreads = 256;
constexpr int kMfmaPerIter = 8;

// Register-resident loop of v_mfma_f32_32x32x16_bf16 (two independent accumulator chains per wave).
__global__ void __launch_bounds__(kDiagThreads)
diag_mfma_kernel(float* __restrict__ sink, int iters) {
  f32x16 acc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = static_cast<bf16_t>(0.5f + 0.001f * (float)(threadIdx.x & 7));
    b[e] = static_cast<bf16_t>(0.25f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < kMfmaPerIter; ++m)
      acc[m & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m & 1], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[(size_t)blockIdx.x * kDiagThreads + threadIdx.x] = s;
}

// Streaming read: every 16-byte piece of [src, src + bytes) is loaded once and folded into a per-thread
// checksum.  Each workgroup walks one contiguous share with eight loads in flight per thread.
__global__ void __launch_bounds__(kDiagThreads)
diag_read_kernel(const u32x4* __restrict__ src, size_t pieces, uint32_t* __restrict__ sink) {
  constexpr int U = 8;
  const size_t share = (pieces + gridDim.x - 1) / gridDim.x;
  const size_t begin = (size_t)blockIdx.x * share;
  const size_t end = begin + share < pieces ? begin + share : pieces;
  uint32_t s = 0;
  for (size_t i = begin + threadIdx.x; i < end; i += (size_t)kDiagThreads * U) {
    u32x4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t j = i + (size_t)u * kDiagThreads;
      // past the share: re-read a piece it already has (not counted) instead of branching.  Non-temporal loads, as
      // the streaming kernels use: they sustain about 7.2 TB/s here where ordinary loads reach 6.0-6.4
      x[u] = __builtin_nontemporal_load(src + (j < end ? j : i));
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      s += (i + (size_t)u * kDiagThreads < end) ? (x[u][0] ^ x[u][1] ^ x[u][2] ^ x[u][3]) : 0u;
  }
  sink[(size_t)blockIdx.x * kDiagThreads + threadIdx.x] = s;
}

}  // namespace
}  // namespace ltea

extern "C" {

size_t ltea_diag_sink_bytes(void) { return (size_t)LTEA_DIAG_BLOCKS * ltea::kDiagThreads * 4; }

int ltea_diag_mfma_loop(int32_t iters, void* sink, double* flops_out, void* stream) {
  if (iters < 1 || !sink) return LTEA_EINVAL;
  hipLaunchKernelGGL(ltea::diag_mfma_kernel, dim3(LTEA_DIAG_BLOCKS), dim3(ltea::kDiagThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<float*>(sink), (int)iters);
  if (hipGetLastError() != hipSuccess) return LTEA_EHIP;
  if (flops_out)
    *flops_out = (double)LTEA_DIAG_BLOCKS * (ltea::kDiagThreads / ltea::kWave) * (double)iters * ltea::kMfmaPerIter *
                 (2.0 * 32 * 32 * 16);
  return LTEA_OK;
}

int ltea_diag_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes == 0 || bytes % 16 != 0 || ((uintptr_t)src & 15)) return LTEA_EINVAL;
  hipLaunchKernelGGL(ltea::diag_read_kernel, dim3(LTEA_DIAG_BLOCKS), dim3(ltea::kDiagThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<const ltea::u32x4*>(src), bytes / 16,
                     static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? LTEA_OK : LTEA_EHIP;
}

}  // extern "C"
