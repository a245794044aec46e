// The one-reflection-at-a-time comparison kernels (Section 2.2) and the log-determinant of Table 1.
// Included by fasth.hip, the library's single translation unit.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// One reflection at a time (Section 2.2): the comparison FastH is measured against.
// One workgroup per column; every reflection costs a workgroup-wide reduction and a barrier.
// ------------------------------------------------------------------------------------------

template <int U>
__global__ void __launch_bounds__(1024) seq_forward_kernel(const float* __restrict__ V, const float* __restrict__ X,
                                                           float* __restrict__ A, int d, int n, int m, int transpose) {
  __shared__ float part[2][16][2];
  const int nthreads = blockDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const int col = blockIdx.x;
  float a[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int x = tid + u * nthreads;
    a[u] = x < d ? X[(size_t)x * m + col] : 0.f;
  }
  // the next reflection's vector is fetched while this one is applied, so that only the inner product, not the
  // trip to memory, lies between two reflections
  float vn[U];
  {
    const float* vr = V + (size_t)(transpose ? 0 : n - 1) * d;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int x = tid + u * nthreads;
      vn[u] = x < d ? vr[x] : 0.f;
    }
  }
  for (int s = 0; s < n; ++s) {
    float v[U];
    float r[2] = {0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) {
      v[u] = vn[u];
      r[0] += v[u] * a[u];
      r[1] += v[u] * v[u];
    }
    if (s + 1 < n) {
      const float* vr = V + (size_t)(transpose ? s + 1 : n - 2 - s) * d;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int x = tid + u * nthreads;
        vn[u] = x < d ? vr[x] : 0.f;
      }
    }
    wave_reduce_multi<2>(r);
    const int sel = reduce_sel<2>(lane);
    if ((lane & reduce_writer_mask<2>()) == 0) part[s & 1][wave][sel] = r[0];
    __syncthreads();
    float va = 0.f, vv = 0.f;
    for (int w = 0; w < nw; ++w) {
      va += part[s & 1][w][0];
      vv += part[s & 1][w][1];
    }
    const float c = 2.f * va / vv;
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] -= c * v[u];
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int x = tid + u * nthreads;
    if (x < d) A[(size_t)x * m + col] = a[u];
  }
}

// Walks the reflections from the output side (Section 3.2 with blocks of one reflection): recovers the
// input of H_j from its output (Eq. 4), emits this column's term of Eq. 5 into dVpart[col][j][:], and
// moves the gradient through H_j.
template <int U>
__global__ void __launch_bounds__(1024) seq_backward_kernel(const float* __restrict__ V, const float* __restrict__ A,
                                                            const float* __restrict__ G, float* __restrict__ dVpart,
                                                            float* __restrict__ dX, int d, int n, int m, int transpose) {
  __shared__ float part[2][16][4];
  const int nthreads = blockDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const int col = blockIdx.x;
  float a[U], g[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int x = tid + u * nthreads;
    a[u] = x < d ? A[(size_t)x * m + col] : 0.f;
    g[u] = x < d ? G[(size_t)x * m + col] : 0.f;
  }
  float vn[U];  // the next reflection's vector, fetched one reflection ahead as in the forward kernel
  {
    const float* vr = V + (size_t)(transpose ? n - 1 : 0) * d;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int x = tid + u * nthreads;
      vn[u] = x < d ? vr[x] : 0.f;
    }
  }
  for (int s = 0; s < n; ++s) {
    const int j = transpose ? n - 1 - s : s;
    float v[U];
    float r[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) {
      v[u] = vn[u];
      r[0] += v[u] * a[u];
      r[1] += v[u] * g[u];
      r[2] += v[u] * v[u];
    }
    if (s + 1 < n) {
      const float* vr = V + (size_t)(transpose ? n - 2 - s : s + 1) * d;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int x = tid + u * nthreads;
        vn[u] = x < d ? vr[x] : 0.f;
      }
    }
    wave_reduce_multi<4>(r);
    const int sel = reduce_sel<4>(lane);
    if ((lane & reduce_writer_mask<4>()) == 0) part[s & 1][wave][sel] = r[0];
    __syncthreads();
    float va = 0.f, vg = 0.f, vv = 0.f;
    for (int w = 0; w < nw; ++w) {
      va += part[s & 1][w][0];
      vg += part[s & 1][w][1];
      vv += part[s & 1][w][2];
    }
    const float t = 2.f / vv;
    const float alpha = -va;  // v^T (input of H_j) = -v^T (output of H_j)
    float* dst = dVpart + ((size_t)col * n + j) * d;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int x = tid + u * nthreads;
      a[u] -= t * va * v[u];  // input of H_j
      if (x < d) dst[x] = -t * (alpha * g[u] + vg * a[u] - t * alpha * vg * v[u]);
      g[u] -= t * vg * v[u];
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int x = tid + u * nthreads;
    if (x < d) dX[(size_t)x * m + col] = g[u];
  }
}

__global__ void __launch_bounds__(256) seq_reduce_kernel(const float* __restrict__ dVpart, float* __restrict__ dV,
                                                         size_t nd, int m) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= nd) return;
  float s = 0.f;
  for (int c = 0; c < m; ++c) s += dVpart[(size_t)c * nd + idx];
  dV[idx] = s;
}

// ------------------------------------------------------------------------------------------
// Table 1, row "Determinant": log|det W| = sum_i log|sigma_i| and its gradient 1/sigma_i. One workgroup,
// fixed summation order.
__global__ void __launch_bounds__(256) logabsdet_kernel(const float* __restrict__ sigma, float* __restrict__ out,
                                                        float* __restrict__ dsigma, int d) {
  __shared__ float part[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float r[1] = {0.f};
  for (int x = tid; x < d; x += 256) {
    const float sg = sigma[x];
    r[0] += logf(fabsf(sg));
    if (dsigma) dsigma[x] = 1.f / sg;
  }
  wave_reduce_multi<1>(r);
  if (lane == 0) part[wave] = r[0];
  __syncthreads();
  if (tid == 0) out[0] = (part[0] + part[1]) + (part[2] + part[3]);
}

}  // namespace fasth
