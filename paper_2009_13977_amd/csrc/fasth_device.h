// Device-side helpers shared by the FastH kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>

namespace fasth {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// One 16x16 output tile of a matrix product on the fp32 matrix cores, operands in LDS.
//   acc(r, c) += sum_{kk < K} A(r, kk) * B(kk, c),   K a multiple of 4
//   A(r, kk) = As[r * sai + kk * sak],  B(kk, c) = Bs[kk * sbk + c * sbj]
// v_mfma_f32_16x16x4_f32 lane layout: lane = 16 q + i supplies A(i, q) and B(q, i) of each
// 4-deep slice and owns acc[j] = tile(4 q + j, i).
__device__ __forceinline__ f32x4 tile_mma(const float* As, int sai, int sak, const float* Bs, int sbk,
                                          int sbj, int K, f32x4 acc) {
  const int lane = threadIdx.x & (kWave - 1);
  const int i = lane & 15, q = lane >> 4;
  const float* ap = As + i * sai + q * sak;
  const float* bp = Bs + q * sbk + i * sbj;
  for (int kk = 0; kk < K; kk += 4) {
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ap[kk * sak], bp[kk * sbk], acc, 0, 0, 0);
  }
  return acc;
}

// Sum NV per-lane values over the 64 lanes of a wave. On return v[0] holds, in every lane, the
// wave-wide sum of the input v[sel] where sel = reduce_sel<NV>(lane); the other entries are scratch.
// Each exchange halves the number of live values, so NV values cost NV - 1 + log2(64 / NV) shuffles.
template <int NV>
__device__ __forceinline__ void wave_reduce_multi(float (&v)[NV]) {
  static_assert(NV == 1 || NV == 2 || NV == 4 || NV == 8 || NV == 16 || NV == 32, "NV must be a power of two");
  const int lane = threadIdx.x & (kWave - 1);
  int mask = 32;
#pragma unroll
  for (int cnt = NV; cnt > 1; cnt >>= 1) {
    const bool upper = (lane & mask) != 0;
#pragma unroll
    for (int idx = 0; idx < cnt / 2; ++idx) {
      const float send = upper ? v[idx] : v[idx + cnt / 2];
      const float keep = upper ? v[idx + cnt / 2] : v[idx];
      v[idx] = keep + __shfl_xor(send, mask, kWave);
    }
    mask >>= 1;
  }
#pragma unroll
  for (; mask >= 1; mask >>= 1) v[0] += __shfl_xor(v[0], mask, kWave);
}

// Index of the input value whose wave-wide sum wave_reduce_multi<NV> leaves in this lane's v[0].
template <int NV>
__device__ __forceinline__ int reduce_sel(int lane) {
  int sel = 0, mask = 32;
#pragma unroll
  for (int cnt = NV; cnt > 1; cnt >>= 1) {
    if (lane & mask) sel += cnt / 2;
    mask >>= 1;
  }
  return sel;
}

// Lanes for which (lane & reduce_writer_mask<NV>()) == 0 are the canonical holders of each sum.
template <int NV>
__device__ __forceinline__ constexpr int reduce_writer_mask() {
  return (kWave / NV) - 1;
}

}  // namespace fasth
