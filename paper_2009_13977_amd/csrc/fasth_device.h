// Device-side helpers shared by the FastH kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>

namespace fasth {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Raised (never cleared) by a kernel whose bounded wait for another workgroup ran out; fasth_wait_status() reads
// and clears it. One word per GPU for the whole library: it says that a launch went wrong, not which.
__device__ unsigned g_wait_gave_up;

constexpr int kWave = 64;

// Buffer addressing: the descriptor (scalar registers) holds base and size; a load takes a per-lane
// byte offset and a scalar byte offset. A lane whose offset lies beyond the buffer (kOob is beyond
// every buffer used here, all < 2 GiB) gets zeros and causes no memory traffic, so bounds checks
// need no branch and the loads of a tile can all be in flight together.
typedef __amdgpu_buffer_rsrc_t BufferDesc;
constexpr unsigned kOob = 0x80000000u;

__device__ __forceinline__ BufferDesc make_buffer(const float* base, size_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), 0, (int)bytes, 0x00020000);
}

// VEC consecutive floats (1 or 4) at byte offset lane_bytes + uniform_bytes of the buffer.
template <int VEC>
struct BufVec {
  float e[VEC];
};
template <int VEC>
__device__ __forceinline__ BufVec<VEC> buffer_load(BufferDesc desc, unsigned lane_bytes, unsigned uniform_bytes) {
  BufVec<VEC> r;
  if constexpr (VEC == 4) {
    const float4 v = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(desc, lane_bytes, uniform_bytes, 0));
    r.e[0] = v.x; r.e[1] = v.y; r.e[2] = v.z; r.e[3] = v.w;
  } else {
    static_assert(VEC == 1, "1 or 4 floats");
    r.e[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(desc, lane_bytes, uniform_bytes, 0));
  }
  return r;
}
// Store of VEC consecutive floats; a lane whose offset lies beyond the buffer stores nothing.
template <int VEC>
__device__ __forceinline__ void buffer_store(BufferDesc desc, unsigned lane_bytes, unsigned uniform_bytes, const BufVec<VEC>& v) {
  if constexpr (VEC == 4) {
    const u32x4 w = {__float_as_uint(v.e[0]), __float_as_uint(v.e[1]), __float_as_uint(v.e[2]), __float_as_uint(v.e[3])};
    __builtin_amdgcn_raw_buffer_store_b128(w, desc, lane_bytes, uniform_bytes, 0);
  } else {
    static_assert(VEC == 1, "1 or 4 floats");
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v.e[0]), desc, lane_bytes, uniform_bytes, 0);
  }
}
template <int VEC>
__device__ __forceinline__ void lds_store(float* dst, const BufVec<VEC>& v) {
  if constexpr (VEC == 4) {
    *reinterpret_cast<float4*>(dst) = make_float4(v.e[0], v.e[1], v.e[2], v.e[3]);
  } else {
    dst[0] = v.e[0];
  }
}

// One 16x16 output tile of a matrix product on the fp32 matrix cores, operands in LDS.
//   acc(r, c) += sum_{kk < K} A(r, kk) * B(kk, c),   K a multiple of 32
//   A(r, kk) = As[r * sai + kk] with 16-byte aligned rows;
//   B(kk, c) = Bs[c * sb + kk] (B_ALONG_K: contiguous along the inner index like A, 16-byte aligned) or Bs[kk * sb + c].
// v_mfma_f32_16x16x4_f32 lane layout: lane = 16 q + i supplies A(i, .) and B(., i) for the q-th of the four inner
// indices of an instruction and owns acc[j] = tile(4 q + j, i). The inner sum may run in any order: of each 16
// inner indices lane (i, q) takes 4 q .. 4 q + 3, one 16-byte read per operand that is contiguous along the inner
// index, and the reads of 32 inner indices are issued ahead of their eight instructions (one trip to LDS per
// instruction otherwise, which is what bounds a short product).
template <bool B_ALONG_K>
__device__ __forceinline__ f32x4 tile_mma(const float* As, int sai, const float* Bs, int sb, int K, f32x4 acc) {
  const int lane = threadIdx.x & (kWave - 1);
  const int i = lane & 15, q = lane >> 4;
  const float* ap = As + i * sai + 4 * q;
  const float* bp = B_ALONG_K ? Bs + i * sb + 4 * q : Bs + 4 * q * sb + i;
  for (int k0 = 0; k0 < K; k0 += 32) {
    float a[8], b[8];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float4 v = *reinterpret_cast<const float4*>(ap + k0 + 16 * h);
      a[4 * h] = v.x; a[4 * h + 1] = v.y; a[4 * h + 2] = v.z; a[4 * h + 3] = v.w;
      if constexpr (B_ALONG_K) {
        const float4 w = *reinterpret_cast<const float4*>(bp + k0 + 16 * h);
        b[4 * h] = w.x; b[4 * h + 1] = w.y; b[4 * h + 2] = w.z; b[4 * h + 3] = w.w;
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) b[4 * h + u] = bp[(k0 + 16 * h + u) * sb];
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u], b[u], acc, 0, 0, 0);
  }
  return acc;
}

// The same product for a compile-time depth K (a multiple of 16) with A contiguous along the inner index
// (16-byte aligned rows) and B contiguous along c: the sum may run in any order, so lane (i, q) takes the inner
// indices q K/4 .. (q + 1) K/4 - 1, its A operands come as 16-byte reads, and every read is issued before the
// first matrix instruction instead of one trip to LDS per 4-deep slice.
template <int K>
__device__ __forceinline__ f32x4 tile_mma_rows(const float* As, int sai, const float* Bs, int sbk, f32x4 acc) {
  static_assert(K % 16 == 0, "four inner indices per 16-byte read and lane group");
  const int lane = threadIdx.x & (kWave - 1);
  const int i = lane & 15, q = lane >> 4;
  constexpr int PER = K / 4;
  float a[PER], b[PER];
#pragma unroll
  for (int g = 0; g < PER / 4; ++g) {
    const float4 v = *reinterpret_cast<const float4*>(As + i * sai + q * PER + 4 * g);
    a[4 * g] = v.x; a[4 * g + 1] = v.y; a[4 * g + 2] = v.z; a[4 * g + 3] = v.w;
  }
#pragma unroll
  for (int kk = 0; kk < PER; ++kk) b[kk] = Bs[(q * PER + kk) * sbk + i];
#pragma unroll
  for (int kk = 0; kk < PER; ++kk) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[kk], b[kk], acc, 0, 0, 0);
  return acc;
}

// Sum NV per-lane values over the 64 lanes of a wave. On return v[0] holds, in every lane, the
// wave-wide sum of the input v[sel] where sel = reduce_sel<NV>(lane); the other entries are scratch.
// Each exchange halves the number of live values, so NV values cost NV - 1 + log2(64 / NV) shuffles.
template <int NV>
__device__ __forceinline__ void wave_reduce_multi(float (&v)[NV]) {
  static_assert(NV == 1 || NV == 2 || NV == 4 || NV == 8 || NV == 16 || NV == 32 || NV == 64, "NV must be a power of two");
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

// Cross-lane moves used by the register-only reduction below.
//   swap32 / swap16: v_permlane32_swap / v_permlane16_swap exchange the odd 32-lane half (16-lane
//   row) of the first operand with the even half (row) of the second, so x + y afterwards is
//   "what I keep + what my partner sent" for both partners at once.
//   dpp_*: DPP row_mirror (lane i <-> 15 - i), row_half_mirror (i <-> 7 - i) and quad permutes
//   (i <-> i ^ 2, i <-> i ^ 1). Each pairs a lane with one whose bit 3 / 2 / 1 / 0 differs.
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float swap32_sum(float keep_lo, float keep_hi) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(keep_lo), __float_as_uint(keep_hi), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float swap16_sum(float keep_lo, float keep_hi) {
  const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(keep_lo), __float_as_uint(keep_hi), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xF, 0xF, false));
}
constexpr int kDppRowMirror = 0x140, kDppRowHalfMirror = 0x141, kDppQuadXor2 = 0x4E, kDppQuadXor1 = 0xB1;
constexpr int kDppRowRor8 = 0x128;  // row_ror:8, lane i <-> i ^ 8 within a row of 16

template <int MASK>
__device__ __forceinline__ float partner_value(float x) {
  if constexpr (MASK == 8) return dpp_move<kDppRowMirror>(x);
  else if constexpr (MASK == 4) return dpp_move<kDppRowHalfMirror>(x);
  else if constexpr (MASK == 2) return dpp_move<kDppQuadXor2>(x);
  else return dpp_move<kDppQuadXor1>(x);
}

// One halving stage of the multi-value reduction: CNT live values -> CNT / 2.
// `hook(t)` is called once before each exchange with a running index t (compile-time after
// unrolling); callers use it to slip independent work (e.g. a prefetch) between the exchanges.
template <int NV, int CNT, int MASK, int T0, typename Hook>
__device__ __forceinline__ void reduce_stage(float (&v)[NV], int lane, Hook& hook) {
  if constexpr (CNT > 1) {
#pragma unroll
    for (int idx = 0; idx < CNT / 2; ++idx) {
      hook(T0 + idx);
      if constexpr (MASK == 32) v[idx] = swap32_sum(v[idx], v[idx + CNT / 2]);
      else if constexpr (MASK == 16) v[idx] = swap16_sum(v[idx], v[idx + CNT / 2]);
      else {
        const bool upper = (lane & MASK) != 0;
        const float send = upper ? v[idx] : v[idx + CNT / 2];
        const float keep = upper ? v[idx + CNT / 2] : v[idx];
        v[idx] = keep + partner_value<MASK>(send);
      }
    }
  } else {
    if constexpr (MASK == 32) v[0] = swap32_sum(v[0], v[0]);
    else if constexpr (MASK == 16) v[0] = swap16_sum(v[0], v[0]);
    else v[0] += partner_value<MASK>(v[0]);
  }
}

struct NoHook {
  __device__ __forceinline__ void operator()(int) const {}
};

// Same contract as wave_reduce_multi (same reduce_sel / reduce_writer_mask), but entirely in
// vector registers: no LDS crossbar traffic. Lanes that share a `sel` may differ in the last
// bits (different summation order), so only the writer lanes' copies are to be used.
template <int NV, typename Hook>
__device__ __forceinline__ void wave_reduce_multi_reg(float (&v)[NV], Hook& hook) {
  static_assert(NV == 1 || NV == 2 || NV == 4 || NV == 8 || NV == 16 || NV == 32 || NV == 64, "power of two");
  const int lane = threadIdx.x & (kWave - 1);
  // exchanges before each stage: NV/2, NV/4, ... (stages with one live value make none)
  reduce_stage<NV, NV, 32, 0>(v, lane, hook);
  reduce_stage<NV, (NV >= 2 ? NV / 2 : 1), 16, NV / 2>(v, lane, hook);
  reduce_stage<NV, (NV >= 4 ? NV / 4 : 1), 8, NV / 2 + NV / 4>(v, lane, hook);
  reduce_stage<NV, (NV >= 8 ? NV / 8 : 1), 4, NV / 2 + NV / 4 + NV / 8>(v, lane, hook);
  reduce_stage<NV, (NV >= 16 ? NV / 16 : 1), 2, NV / 2 + NV / 4 + NV / 8 + NV / 16>(v, lane, hook);
  reduce_stage<NV, (NV >= 32 ? NV / 32 : 1), 1, NV / 2 + NV / 4 + NV / 8 + NV / 16 + NV / 32>(v, lane, hook);
}

template <int NV>
__device__ __forceinline__ void wave_reduce_multi_reg(float (&v)[NV]) {
  NoHook h;
  wave_reduce_multi_reg<NV>(v, h);
}

// Sum over groups of G consecutive lanes (G = 4, 8 or 16); every lane of the group gets the total.
template <int G>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_move<kDppQuadXor1>(x);
  x += dpp_move<kDppQuadXor2>(x);
  if constexpr (G >= 8) x += dpp_move<kDppRowHalfMirror>(x);
  if constexpr (G >= 16) x += dpp_move<kDppRowMirror>(x);
  return x;
}

// Barrier that orders LDS traffic only: global loads issued earlier (prefetches) stay in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
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
