// Benchmark aid: what this GPU delivers on the two rooflines the FastH kernels are priced against, measured with
// plain kernels of known work (fp32 matrix instructions from registers; a streaming read and a copy of a large
// buffer). Included by fasth.hip, the library's single translation unit.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

constexpr int kPeakMfmaPerIter = 8;  // independent accumulators per wave

// Every wave issues iters x 8 v_mfma_f32_16x16x4_f32 (2048 FLOP each) on independent accumulators.
__global__ void __launch_bounds__(256) peak_mfma_kernel(float* __restrict__ out, int iters) {
  const float a = 1.0f + 1e-3f * (float)threadIdx.x, b = 1.0f - 1e-3f * (float)threadIdx.x;
  f32x4 c[kPeakMfmaPerIter];
#pragma unroll
  for (int u = 0; u < kPeakMfmaPerIter; ++u) c[u] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < kPeakMfmaPerIter; ++u) c[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c[u], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < kPeakMfmaPerIter; ++u) s += c[u][0] + c[u][1] + c[u][2] + c[u][3];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Grid-stride read of `count` 16-byte pieces; one float per workgroup is written so that the reads are kept.
__global__ void __launch_bounds__(256) peak_read_kernel(const float4* __restrict__ src, size_t count, float* __restrict__ out) {
  float s = 0.f;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) {
    const float4 v = src[i];
    s += (v.x + v.y) + (v.z + v.w);
  }
  float r[1] = {s};
  wave_reduce_multi<1>(r);
  if ((threadIdx.x & 63) == 0) out[(size_t)blockIdx.x * 4 + (threadIdx.x >> 6)] = r[0];
}

__global__ void __launch_bounds__(256) peak_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t count) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) dst[i] = src[i];
}

}  // namespace fasth
