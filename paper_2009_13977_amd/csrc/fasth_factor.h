// Algorithm 1 Step 1: the k x k block factors T_i (gram_partial_kernel + t_build_kernel, factor_fused_kernel).
// Included by fasth.hip, the library's single translation unit.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// Algorithm 1 Step 1a: partial Gram matrices S_i = V_i V_i^T, split over d.
// grid (gram_split, nb), 256 threads. Only the 16x16 tiles on or above the diagonal are formed.
// ------------------------------------------------------------------------------------------

// The hand-off area of the workspace (words that workgroups of a later chain launch pass to each other, with the
// counters their tags continue from) starts every product at zero: whichever kernel builds the factors clears it,
// all its workgroups taking a share.
__device__ __forceinline__ void clear_exchange_area(unsigned* xch, unsigned words, unsigned wg, unsigned wgs) {
  // the area is 256-byte aligned and a whole number of 16-byte pieces
  u32x4* x4 = reinterpret_cast<u32x4*>(xch);
  for (unsigned w = wg * blockDim.x + threadIdx.x; w < words / 4u; w += wgs * blockDim.x) x4[w] = u32x4{0u, 0u, 0u, 0u};
}

template <int VEC>  // VEC = 4 when d is a multiple of 4 (16-byte loads), else 1
__global__ void __launch_bounds__(256) gram_partial_kernel(const float* __restrict__ V, float* __restrict__ Spart,
                                                           int d, int k, int kp, int gram_split, unsigned* xch,
                                                           unsigned xch_words) {
  extern __shared__ __align__(16) float smem[];
  const int LD = kGramChunk + 4;
  float* Vs = smem;  // [kp][LD]
  const int i = blockIdx.y, s = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  clear_exchange_area(xch, xch_words, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
  const int chunk = ((d + gram_split - 1) / gram_split + 3) & ~3;
  const int xbeg = s * chunk;
  const int xend = min(d, xbeg + chunk);
  const int kt = kp / 16;
  const int ntiles = kt * (kt + 1) / 2;
  constexpr int kMaxTilesPerWave = 9;  // kp = 128: 36 upper tiles over 4 waves
  f32x4 acc[kMaxTilesPerWave];
#pragma unroll
  for (int w = 0; w < kMaxTilesPerWave; ++w) acc[w] = f32x4{0.f, 0.f, 0.f, 0.f};
  // the block's k rows as one buffer: rows k .. kp - 1 of the padded block lie beyond it and read as zero
  const BufferDesc vdesc = make_buffer(V + (size_t)i * k * d, (size_t)k * d * sizeof(float));
  constexpr int XV = kGramChunk / VEC;             // loads per slab row
  constexpr int kMaxPer = kMaxBlock * XV / 256;    // loads per thread and slab at the largest block
  const int per = kp * XV / 256;
  for (int x0 = xbeg; x0 < xend; x0 += kGramChunk) {
    BufVec<VEC> stage[kMaxPer];
#pragma unroll
    for (int it = 0; it < kMaxPer; ++it) {
      if (it < per) {  // uniform
        const int idx = tid + it * 256, j = idx / XV, x = x0 + (idx % XV) * VEC;
        stage[it] = buffer_load<VEC>(vdesc, x < xend ? (unsigned)(j * d + x) * 4u : kOob, 0);
      }
    }
#pragma unroll
    for (int it = 0; it < kMaxPer; ++it) {
      if (it < per) {
        const int idx = tid + it * 256;
        lds_store<VEC>(Vs + (idx / XV) * LD + (idx % XV) * VEC, stage[it]);
      }
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kMaxTilesPerWave; ++w) {
      const int t = wave + 4 * w;
      if (t < ntiles) {
        int ti = 0, rem = t;
        while (rem >= kt - ti) { rem -= kt - ti; ++ti; }
        const int tj = ti + rem;
        acc[w] = tile_mma<true>(Vs + ti * 16 * LD, LD, Vs + tj * 16 * LD, LD, kGramChunk, acc[w]);
      }
    }
    __syncthreads();
  }
  float* out = Spart + ((size_t)i * gram_split + s) * kp * kp;
  const int li = lane & 15, q = lane >> 4;
#pragma unroll
  for (int w = 0; w < kMaxTilesPerWave; ++w) {
    const int t = wave + 4 * w;
    if (t < ntiles) {
      int ti = 0, rem = t;
      while (rem >= kt - ti) { rem -= kt - ti; ++ti; }
      const int tj = ti + rem;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) out[(ti * 16 + 4 * q + jj) * kp + tj * 16 + li] = acc[w][jj];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Algorithm 1 Step 1b: T_i = (diag(S)/2 + striu(S))^-1, one workgroup per block.
// 16x16 diagonal blocks by unrolled back substitution, then [[T11, -T11 M12 T22], [0, T22]] doubles
// the block size each level with matrix-core products. Rows/columns >= k (padding) form an identity.
// ------------------------------------------------------------------------------------------

// Floats of LDS scratch that invert_upper_lds needs beside the matrix.
__host__ __device__ constexpr int invert_scratch_floats(int kp) {
  return kp * (kp / 2 + 4) / 2 + 64 > kp * 21 ? kp * (kp / 2 + 4) / 2 + 64 : kp * 21;
}

// The inversion reads the 16 x 16 diagonal blocks from a copy in the scratch: rows of kDiagLd floats, which a
// solving thread reads four entries at a time, followed by the reciprocals of the diagonal (one division per
// entry, by whoever stores it, off the dependent chain of the solve).
constexpr int kDiagLd = 20;
__device__ __forceinline__ void diag_scratch_store(float* Xs, int kp, int j, int l, float v) {
  if ((j ^ l) < 16) {  // same diagonal block
    Xs[j * kDiagLd + (l & 15)] = v;
    if (j == l) Xs[kp * kDiagLd + j] = 1.f / v;
  }
}

// Fills that copy from a complete Ms; ends with a barrier.
__device__ __forceinline__ void diag_scratch_fill(const float* Ms, float* Xs, int kp, int LDM) {
  for (int idx = threadIdx.x; idx < kp * 16; idx += blockDim.x) {
    const int r = idx >> 4, c = idx & 15;
    diag_scratch_store(Xs, kp, r, (r & ~15) + c, Ms[r * LDM + (r & ~15) + c]);
  }
  __syncthreads();
}

// In-place inverse of the upper-triangular kp x kp matrix Ms (row stride LDM, a multiple of 4; Ms 16-byte
// aligned) in LDS by block doubling; Xs is 16-byte aligned scratch of invert_scratch_floats(kp) floats that
// holds the copy of the diagonal blocks on entry (diag_scratch_fill, or diag_scratch_store by whoever builds
// Ms). Called by every thread of the workgroup (a multiple of 64 threads); Ms and the copy must be complete
// (barrier) on entry and Ms is complete on return.
// PRELOAD: a solving thread fetches all it reads of its diagonal block (144 registers) before the first row
// instead of row by row, and works column by column; for kernels whose register budget allows it. Both orders
// give the same bits.
template <bool PRELOAD>
__device__ __forceinline__ void invert_upper_lds(float* Ms, float* Xs, int kp, int LDM) {
  const int tid = threadIdx.x, nthreads = blockDim.x, wave = tid >> 6, nwaves = nthreads >> 6, lane = tid & 63;
  const int li = lane & 15, q = lane >> 4;
  // 16x16 diagonal blocks: thread c of a block solves for column c by back substitution, fully unrolled so
  // that the reads of M are independent of the values being computed (every thread of a block reads the same
  // addresses).
  if (tid < kp) {
    const int base = tid & ~15, c = tid & 15;
    const float4* D4 = reinterpret_cast<const float4*>(Xs + base * kDiagLd);
    const float4* R4 = reinterpret_cast<const float4*>(Xs + kp * kDiagLd + base);
    float x[16], rdiag[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 v = R4[g];
      rdiag[4 * g] = v.x; rdiag[4 * g + 1] = v.y; rdiag[4 * g + 2] = v.z; rdiag[4 * g + 3] = v.w;
    }
    if constexpr (PRELOAD) {
      // column by column: once x[l] is known it leaves every row's sum above it, products that do not depend
      // on one another; only one multiply-add and one multiply per row lie on the dependent chain. Each sum
      // still takes its terms oldest x first, as below.
      float row[16][16], sum[16];
#pragma unroll
      for (int r = 15; r >= 0; --r) {
#pragma unroll
        for (int g = (r + 1) / 4; g < 4; ++g) {
          const float4 v = D4[r * (kDiagLd / 4) + g];
          row[r][4 * g] = v.x; row[r][4 * g + 1] = v.y; row[r][4 * g + 2] = v.z; row[r][4 * g + 3] = v.w;
        }
        sum[r] = r == c ? 1.f : 0.f;
      }
#pragma unroll
      for (int l = 15; l >= 0; --l) {
        x[l] = sum[l] * rdiag[l];  // rows below c stay exactly zero
#pragma unroll
        for (int r = l - 1; r >= 0; --r) sum[r] = fmaf(-row[r][l], x[l], sum[r]);
      }
    } else {
#pragma unroll
      for (int r = 15; r >= 0; --r) {
        float row[16];
#pragma unroll
        for (int g = (r + 1) / 4; g < 4; ++g) {
          const float4 v = D4[r * (kDiagLd / 4) + g];
          row[4 * g] = v.x; row[4 * g + 1] = v.y; row[4 * g + 2] = v.z; row[4 * g + 3] = v.w;
        }
        float sum = r == c ? 1.f : 0.f;
        // oldest x first: the value computed last enters last, so each row adds one multiply-add to the chain
#pragma unroll
        for (int l = 15; l > r; --l) sum = fmaf(-row[l], x[l], sum);
        x[r] = sum * rdiag[r];  // rows below c stay exactly zero
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) Ms[(base + r) * LDM + base + c] = x[r];
  }
  __syncthreads();
  // [[T11, -T11 M12 T22], [0, T22]] for pairs of 16 x 16 blocks, one wave per pair and both products in
  // registers: product j of X = M12 T22 sums over the inner indices 4 q + j, for which lane (i, q) supplies
  // M12(i, 4 q + j) and T22(4 q + j, i); the lane then owns X(4 q + j, i), which is exactly the operand that
  // product j of T11 X wants from it.
  if (kp >= 32) {
    for (int pr = wave; pr < kp / 32; pr += nwaves) {
      const int r0 = pr * 32;
      const float4 m12 = *reinterpret_cast<const float4*>(Ms + (r0 + li) * LDM + r0 + 16 + 4 * q);
      const float4 t11 = *reinterpret_cast<const float4*>(Ms + (r0 + li) * LDM + r0 + 4 * q);
      float t22[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) t22[jj] = Ms[(r0 + 16 + 4 * q + jj) * LDM + r0 + 16 + li];
      f32x4 X = {0.f, 0.f, 0.f, 0.f};
      X = __builtin_amdgcn_mfma_f32_16x16x4f32(m12.x, t22[0], X, 0, 0, 0);
      X = __builtin_amdgcn_mfma_f32_16x16x4f32(m12.y, t22[1], X, 0, 0, 0);
      X = __builtin_amdgcn_mfma_f32_16x16x4f32(m12.z, t22[2], X, 0, 0, 0);
      X = __builtin_amdgcn_mfma_f32_16x16x4f32(m12.w, t22[3], X, 0, 0, 0);
      f32x4 R = {0.f, 0.f, 0.f, 0.f};
      R = __builtin_amdgcn_mfma_f32_16x16x4f32(t11.x, X[0], R, 0, 0, 0);
      R = __builtin_amdgcn_mfma_f32_16x16x4f32(t11.y, X[1], R, 0, 0, 0);
      R = __builtin_amdgcn_mfma_f32_16x16x4f32(t11.z, X[2], R, 0, 0, 0);
      R = __builtin_amdgcn_mfma_f32_16x16x4f32(t11.w, X[3], R, 0, 0, 0);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) Ms[(r0 + 4 * q + jj) * LDM + r0 + 16 + li] = -R[jj];
    }
    __syncthreads();
  }
  for (int b = 32; b < kp; b *= 2) {
    const int tpb = b / 16, per_pair = tpb * tpb, items = (kp / (2 * b)) * per_pair;
    const int LDX = b + 4;
    for (int it = wave; it < items; it += nwaves) {  // X = M12 T22
      const int pr = it / per_pair, ti = (it % per_pair) / tpb, tj = it % tpb, r0 = pr * 2 * b;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = tile_mma<false>(Ms + (r0 + 16 * ti) * LDM + r0 + b, LDM, Ms + (r0 + b) * LDM + r0 + b + 16 * tj, LDM, b, acc);
      float* X = Xs + pr * b * LDX;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) X[(16 * ti + 4 * q + jj) * LDX + 16 * tj + li] = acc[jj];
    }
    __syncthreads();
    for (int it = wave; it < items; it += nwaves) {  // T12 = -T11 X
      const int pr = it / per_pair, ti = (it % per_pair) / tpb, tj = it % tpb, r0 = pr * 2 * b;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = tile_mma<false>(Ms + (r0 + 16 * ti) * LDM + r0, LDM, Xs + pr * b * LDX + 16 * tj, LDX, b, acc);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) Ms[(r0 + 16 * ti + 4 * q + jj) * LDM + r0 + b + 16 * tj + li] = -acc[jj];
    }
    __syncthreads();
  }
}

__global__ void __launch_bounds__(1024) t_build_kernel(const float* __restrict__ Spart, float* __restrict__ T,
                                                      int k, int kp, int gram_split) {
  extern __shared__ __align__(16) float smem[];
  const int LDM = kp + 4;
  float* Ms = smem;                 // [kp][LDM]
  float* Xs = Ms + kp * LDM;        // scratch of the inversion
  const int i = blockIdx.x;
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const float* Sp = Spart + (size_t)i * gram_split * kp * kp;
  // Four neighbouring entries of a row at a time (kp is a multiple of 16, so they share a 16 x 16 tile); tiles
  // below the diagonal hold nothing and are not read. All partial sums of an entry are in flight at once.
  for (int idx4 = tid; idx4 < kp * kp / 4; idx4 += nthreads) {
    const int j = idx4 / (kp / 4), l0 = (idx4 % (kp / 4)) * 4;
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j / 16 <= l0 / 16 && j < k) {
      float4 part[kMaxGramSplit];
#pragma unroll
      for (int s = 0; s < kMaxGramSplit; ++s)
        part[s] = s < gram_split ? *reinterpret_cast<const float4*>(Sp + (size_t)s * kp * kp + 4 * (size_t)idx4)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int s = 0; s < kMaxGramSplit; ++s) {
        sum.x += part[s].x; sum.y += part[s].y; sum.z += part[s].z; sum.w += part[s].w;
      }
    }
    const float e[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int l = l0 + u;
      float v = 0.f;
      if (j < k && l < k && j <= l) v = j == l ? 0.5f * e[u] : e[u];
      else if (j == l) v = 1.f;
      Ms[j * LDM + l] = v;
    }
  }
  __syncthreads();
  diag_scratch_fill(Ms, Xs, kp, LDM);
  invert_upper_lds<false>(Ms, Xs, kp, LDM);
  // T_i and, nb factors further on, its transpose: a chain kernel then reads rows of op(T_i) in either direction
  float* Ti = T + (size_t)i * kp * kp;
  float* Tti = Ti + (size_t)gridDim.x * kp * kp;
  for (int idx = tid; idx < kp * kp; idx += nthreads) {
    Ti[idx] = Ms[(idx / kp) * LDM + idx % kp];
    Tti[idx] = Ms[(idx % kp) * LDM + idx / kp];
  }
}

// Algorithm 1 Step 1 in one kernel for blocks of up to 64 rows (kp = 16 KT): one workgroup of 8 waves per
// block streams the block's rows through LDS in 128-column slabs; wave w multiplies columns
// [16 w, 16 w + 16) of each slab, the 8 partial Gram matrices are added through LDS, and the same
// workgroup inverts. Saves a launch and the round trip of the partial sums through memory.
// Up to two products (the two orthogonal factors of an SVD layer) are factored by one launch:
// blockIdx.y picks the product, blockIdx.x its block.
struct FactorPair {
  const float* V[2];  // [n][d]
  float* T[2];        // [2][nb][kp][kp]: the factors, then their transposes
  int d[2], k[2], nb[2];
  unsigned* xch[2];   // hand-off area of the product's workspace, cleared here
  unsigned xch_words[2];
};

template <int KT, int VEC>  // VEC = 4 when d is a multiple of 4 (16-byte loads), else 1
__global__ void __launch_bounds__(512) factor_fused_kernel(FactorPair fp) {
  const int which = blockIdx.y;
  if ((int)blockIdx.x >= fp.nb[which]) return;  // whole workgroup, before any barrier
  clear_exchange_area(fp.xch[which], fp.xch_words[which], blockIdx.x, fp.nb[which]);
  const float* __restrict__ V = fp.V[which];
  float* __restrict__ T = fp.T[which];
  const int d = fp.d[which], k = fp.k[which];
  constexpr int kp = 16 * KT, LD = kGramChunk + 4, NTILE = KT * (KT + 1) / 2, NW = 8, LDM = kp + 4;
  constexpr int PER = kp * kGramChunk / 512 / VEC;  // loads per thread and slab
  constexpr int XV = kGramChunk / VEC;              // loads per slab row
  // Partial Gram matrices meet in LDS. Up to 32 rows all eight waves' tiles fit side by side; for 64 rows
  // (10 tiles a wave) the upper four waves hand theirs to the lower four first, which halves the space.
  constexpr int RW = KT <= 2 ? NW : NW / 2;  // waves whose partial tiles are held at once
  __shared__ __align__(16) float Vs2[2][kp * LD];  // slabs alternate between the two: one barrier per slab
  __shared__ float Red[RW * NTILE * 256];
  __shared__ __align__(16) float Ms[kp * LDM];
  __shared__ __align__(16) float Xs[invert_scratch_floats(kp)];
  const int i = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, q = lane >> 4;
  // the block's k rows as one buffer: rows k .. kp - 1 of the padded block lie beyond it and read as zero
  const BufferDesc vdesc = make_buffer(V + (size_t)i * k * d, (size_t)k * d * sizeof(float));
  f32x4 acc[NTILE];
#pragma unroll
  for (int t = 0; t < NTILE; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  // Eight slabs (1024 columns) are fetched at once, so the trip to memory is paid once per 1024
  // columns of V instead of once per slab.
  constexpr int NS = 8;
  BufVec<VEC> stage[NS][PER];
  for (int xs = 0; xs < d; xs += NS * kGramChunk) {
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
#pragma unroll
      for (int it = 0; it < PER; ++it) {
        const int idx = tid + it * 512, j = idx / XV, x = xs + sl * kGramChunk + (idx % XV) * VEC;
        stage[sl][it] = buffer_load<VEC>(vdesc, x < d ? (unsigned)(j * d + x) * 4u : kOob, 0);
      }
    }
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
      if (xs + sl * kGramChunk < d) {  // uniform across the workgroup
        // A wave that writes this buffer has passed the barrier of the slab before, which every wave reaches
        // only after its reads of the slab before that one, the buffer's last user.
        float* Vs = Vs2[sl & 1];
#pragma unroll
        for (int it = 0; it < PER; ++it) {
          const int idx = tid + it * 512;
          lds_store<VEC>(Vs + (idx / XV) * LD + (idx % XV) * VEC, stage[sl][it]);
        }
        __syncthreads();
        // This wave's 16 columns of the slab, one 16-byte read per 16-row group: lane (i, q) holds
        // columns 4 q .. 4 q + 3 of row i, which serves as the A fragment of row group ti and as the
        // B fragment of row group tj alike (the matrix cores sum over q; product u takes element u).
        float4 frag[KT];
#pragma unroll
        for (int tt = 0; tt < KT; ++tt)
          frag[tt] = *reinterpret_cast<const float4*>(Vs + (16 * tt + li) * LD + 16 * wave + 4 * q);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          int t = 0;
#pragma unroll
          for (int ti = 0; ti < KT; ++ti) {
            const float av = u == 0 ? frag[ti].x : u == 1 ? frag[ti].y : u == 2 ? frag[ti].z : frag[ti].w;
#pragma unroll
            for (int tj = ti; tj < KT; ++tj) {
              const float bv = u == 0 ? frag[tj].x : u == 1 ? frag[tj].y : u == 2 ? frag[tj].z : frag[tj].w;
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[t], 0, 0, 0);
              ++t;
            }
          }
        }
      }
    }
  }
  if constexpr (RW == NW) {
#pragma unroll
    for (int t = 0; t < NTILE; ++t) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) Red[(wave * NTILE + t) * 256 + (4 * q + jj) * 16 + li] = acc[t][jj];
    }
  } else {
    if (wave >= RW) {
#pragma unroll
      for (int t = 0; t < NTILE; ++t) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) Red[((wave - RW) * NTILE + t) * 256 + (4 * q + jj) * 16 + li] = acc[t][jj];
      }
    }
    __syncthreads();
    if (wave < RW) {
#pragma unroll
      for (int t = 0; t < NTILE; ++t) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) acc[t][jj] += Red[(wave * NTILE + t) * 256 + (4 * q + jj) * 16 + li];
      }
    }
    __syncthreads();
    if (wave < RW) {
#pragma unroll
      for (int t = 0; t < NTILE; ++t) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) Red[(wave * NTILE + t) * 256 + (4 * q + jj) * 16 + li] = acc[t][jj];
      }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < kp * kp; idx += 512) {
    const int j = idx / kp, l = idx % kp;
    float v = 0.f;
    if (j < k && l < k && j <= l) {
      const int ti = j / 16, tj = l / 16;
      const int t = ti * KT - ti * (ti - 1) / 2 + (tj - ti);  // index of tile (ti, tj) in the upper-triangle order
#pragma unroll
      for (int w = 0; w < RW; ++w) v += Red[(w * NTILE + t) * 256 + (j % 16) * 16 + l % 16];
      if (j == l) v *= 0.5f;
    } else if (j == l) {
      v = 1.f;
    }
    Ms[j * LDM + l] = v;
    diag_scratch_store(Xs, kp, j, l, v);
  }
  __syncthreads();
  invert_upper_lds<true>(Ms, Xs, kp, LDM);
  // T_i and, nb factors further on, its transpose: a chain kernel then reads rows of op(T_i) in either direction
  float* Ti = T + (size_t)i * kp * kp;
  float* Tti = Ti + (size_t)fp.nb[which] * kp * kp;
  for (int idx = tid; idx < kp * kp; idx += 512) {
    Ti[idx] = Ms[(idx / kp) * LDM + idx % kp];
    Tti[idx] = Ms[(idx % kp) * LDM + idx / kp];
  }
}

// ------------------------------------------------------------------------------------------
// Blocks of 32 rows merged in pairs (for the chain kernel whose steps take 64 rows). By Lemma 1 the product of
// blocks 2 p and 2 p + 1 is a WY block of 64 rows with the factor
//   T = [[T1, -T1 S12 T2], [0, T2]],   S12 = V_{2p} V_{2p+1}^T,
// T1 and T2 the blocks' own factors (the inverse of [[M1, S12], [0, M2]] with M = diag(S)/2 + striu(S)). A 64-row
// Gram product on one compute unit would take three times as long as a 32-row one, so the work is spread: one
// workgroup per block builds T1 or T2 exactly as factor_fused_kernel does and writes it into the diagonal of the
// pair's 64 x 64 factor (and of its transpose); one workgroup per pair forms S12 (four 16 x 16 tiles instead of
// three), then waits for the pair's two factors, multiplies the corner -T1 S12 T2 out and writes it with the zero
// corner opposite. The block workgroups come first in the launch, so they run (or have run) whenever a pair's
// workgroup waits. "Ready" is an 8-byte word per block that its workgroup sets, after a release fence, to a number
// the host draws anew for every launch; the pair's workgroup clears both words once it has read the factors, so a
// captured launch that is replayed with the same number starts from cleared words again. (A workspace that has
// never been used holds arbitrary words: the chance that one equals the launch's 64-bit number is 2^-64.) The wait
// is bounded like every wait between workgroups in this library: after wait_limit polls the workgroup raises the
// status word and goes on.
// ------------------------------------------------------------------------------------------
constexpr int kPairRows = 64;

// One workgroup's Gram tiles over all of d: CROSS = false: the block's own 32 x 32 (tiles (0,0), (0,1), (1,1) in
// acc[0], acc[1], acc[3]); CROSS = true: rows 0..31 against rows 32..63 of the pair (tile (ti, tj) in acc[2 ti + tj]).
template <int VEC, bool CROSS>
__device__ __forceinline__ void pair_gram_tiles(const BufferDesc vdesc, int d, float* Vs2, f32x4 (&acc)[4]) {
  constexpr int LD = kGramChunk + 4, ROWS = CROSS ? kPairRows : 32, RT = ROWS / 16;
  constexpr int XV = kGramChunk / VEC;                 // loads per slab row
  constexpr int PER = ROWS * kGramChunk / 512 / VEC;   // loads per thread and slab
  constexpr int NS = 8;                                // slabs fetched at once (1024 columns)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, q = lane >> 4;
  BufVec<VEC> stage[NS][PER];
  for (int xs = 0; xs < d; xs += NS * kGramChunk) {
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
#pragma unroll
      for (int it = 0; it < PER; ++it) {
        const int idx = tid + it * 512, j = idx / XV, x = xs + sl * kGramChunk + (idx % XV) * VEC;
        stage[sl][it] = buffer_load<VEC>(vdesc, x < d ? (unsigned)(j * d + x) * 4u : kOob, 0);
      }
    }
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
      if (xs + sl * kGramChunk < d) {  // uniform across the workgroup
        // slabs alternate between two buffers: a wave that writes one has passed the barrier of the slab before,
        // which every wave reaches only after its reads of the slab before that, the buffer's last user
        float* Vs = Vs2 + (sl & 1) * (kPairRows * LD);
#pragma unroll
        for (int it = 0; it < PER; ++it) {
          const int idx = tid + it * 512;
          lds_store<VEC>(Vs + (idx / XV) * LD + (idx % XV) * VEC, stage[sl][it]);
        }
        __syncthreads();
        // this wave's 16 columns of the slab: lane (i, q) holds columns 4 q .. 4 q + 3 of row i of a 16-row group,
        // A fragment and B fragment alike (the matrix cores sum over q; product u takes element u)
        float4 frag[RT];
#pragma unroll
        for (int tt = 0; tt < RT; ++tt) frag[tt] = *reinterpret_cast<const float4*>(Vs + (16 * tt + li) * LD + 16 * wave + 4 * q);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          auto el = [&](const float4& f) { return u == 0 ? f.x : u == 1 ? f.y : u == 2 ? f.z : f.w; };
          if constexpr (CROSS) {
#pragma unroll
            for (int ti = 0; ti < 2; ++ti)
#pragma unroll
              for (int tj = 0; tj < 2; ++tj)
                acc[2 * ti + tj] = __builtin_amdgcn_mfma_f32_16x16x4f32(el(frag[ti]), el(frag[2 + tj]), acc[2 * ti + tj], 0, 0, 0);
          } else {
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(el(frag[0]), el(frag[0]), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(el(frag[0]), el(frag[1]), acc[1], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(el(frag[1]), el(frag[1]), acc[3], 0, 0, 0);
          }
        }
      }
    }
  }
}

template <int VEC>
__global__ void __launch_bounds__(512) pair_factor_kernel(FactorPair fp, unsigned long long* __restrict__ ready0,
                                                          unsigned long long* __restrict__ ready1,
                                                          unsigned long long launch_id, int wait_limit) {
  const int which = blockIdx.y;
  const int nb = fp.nb[which];            // 64-row factors; 2 nb blocks of 32 rows, then nb cross products
  if ((int)blockIdx.x >= 3 * nb) return;  // whole workgroup, before any barrier
  clear_exchange_area(fp.xch[which], fp.xch_words[which], blockIdx.x, 3 * nb);
  const float* __restrict__ V = fp.V[which];
  float* __restrict__ T = fp.T[which];
  const int d = fp.d[which];
  constexpr int LD = kGramChunk + 4, NW = 8, kp = 32, LDM = kp + 4;
  __shared__ __align__(16) float Vs2[2 * kPairRows * LD];
  __shared__ float Red[NW * 4 * 256];
  __shared__ __align__(16) float Ms[kp * LDM];
  __shared__ __align__(16) float Xs[invert_scratch_floats(kp)];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, q = lane >> 4;
  const bool cross = (int)blockIdx.x >= 2 * nb;
  const int i = cross ? (int)blockIdx.x - 2 * nb : (int)blockIdx.x;  // pair, or block of 32
  const int rows = cross ? kPairRows : kp;
  const BufferDesc vdesc = make_buffer(V + (size_t)i * rows * d, (size_t)rows * d * sizeof(float));
  f32x4 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (cross) pair_gram_tiles<VEC, true>(vdesc, d, Vs2, acc);
  else pair_gram_tiles<VEC, false>(vdesc, d, Vs2, acc);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) Red[(wave * 4 + t) * 256 + (4 * q + jj) * 16 + li] = acc[t][jj];
  }
  __syncthreads();
  // element (j, l) of the 32 x 32 result lies in tile 2 (j / 16) + l / 16
  auto summed = [&](int j, int l) {
    const int t = 2 * (j / 16) + l / 16;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) v += Red[(w * 4 + t) * 256 + (j % 16) * 16 + l % 16];
    return v;
  };
  unsigned long long* ready = which == 0 ? ready0 : ready1;  // [2 nb], one word per block of 32 rows
  if (cross) {
    // S12 into LDS (the space of the matrix to invert and, for T1 and T2 and the product S12 T2, of the slabs)
    constexpr int LDP = kp + 1;
    float* S = Ms;  // kp * LDM >= kp * LDP
    float* T1 = Vs2, *T2 = Vs2 + kp * LDP, *Y = Vs2 + 2 * kp * LDP;
    for (int idx = tid; idx < kp * kp; idx += 512) S[(idx / kp) * LDP + idx % kp] = summed(idx / kp, idx % kp);
    // wait for the two blocks' factors
    bool gave_up = false;
    if (wave == 0) {
      const BufferDesc rdesc = make_buffer(reinterpret_cast<const float*>(ready + 2 * i), 16);
      int polls = 0;
      for (;;) {
        const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rdesc, (unsigned)(lane & 1) * 8u, 0, 16);
        const unsigned long long v = ((unsigned long long)w.y << 32) | w.x;
        if (__all(v == launch_id)) break;
        if (polls++ >= wait_limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(2);
        asm volatile("" ::: "memory");
      }
      if (gave_up && lane == 0) __hip_atomic_store(&g_wait_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    float* Tp = T + (size_t)i * kPairRows * kPairRows;
    float* Ttp = Tp + (size_t)nb * kPairRows * kPairRows;
    {
      // the factors as their workgroups wrote them (loads that go past this unit's and this XCD's caches)
      const BufferDesc tdesc = make_buffer(Tp, kPairRows * kPairRows * sizeof(float));
      for (int idx = tid; idx < kp * kp; idx += 512) {
        const int j = idx / kp, l = idx % kp;
        T1[j * LDP + l] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(tdesc, (unsigned)(j * kPairRows + l) * 4u, 0, 16));
        T2[j * LDP + l] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(tdesc, (unsigned)((kp + j) * kPairRows + kp + l) * 4u, 0, 16));
      }
    }
    __syncthreads();
    if (tid == 0) {  // both factors are in LDS: the words can be cleared for the next launch
      ready[2 * i] = 0ull;
      ready[2 * i + 1] = 0ull;
    }
    const int r = tid / 16, c0 = (tid % 16) * 2;  // two entries of a row per thread
    float y0 = 0.f, y1 = 0.f;
    for (int kk = 0; kk < kp; ++kk) {
      const float sv = S[r * LDP + kk];
      y0 = fmaf(sv, T2[kk * LDP + c0], y0);
      y1 = fmaf(sv, T2[kk * LDP + c0 + 1], y1);
    }
    Y[r * LDP + c0] = y0; Y[r * LDP + c0 + 1] = y1;
    __syncthreads();
    float x0 = 0.f, x1 = 0.f;
    for (int kk = 0; kk < kp; ++kk) {
      const float tv = T1[r * LDP + kk];
      x0 = fmaf(tv, Y[kk * LDP + c0], x0);
      x1 = fmaf(tv, Y[kk * LDP + c0 + 1], x1);
    }
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int c = c0 + e;
      const float x = e == 0 ? -x0 : -x1;
      Tp[r * kPairRows + kp + c] = x;
      Tp[(kp + r) * kPairRows + c] = 0.f;
      Ttp[(kp + c) * kPairRows + r] = x;
      Ttp[r * kPairRows + kp + c] = 0.f;
    }
    return;
  }
  for (int idx = tid; idx < kp * kp; idx += 512) {
    const int j = idx / kp, l = idx % kp;
    float v = 0.f;
    if (j <= l) {
      v = summed(j, l);
      if (j == l) v *= 0.5f;
    }
    Ms[j * LDM + l] = v;
    diag_scratch_store(Xs, kp, j, l, v);
  }
  __syncthreads();
  invert_upper_lds<true>(Ms, Xs, kp, LDM);
  // into the diagonal of the pair's 64 x 64 factor and of its transpose (nb factors further on)
  const int h = i & 1;
  float* Tp = T + (size_t)(i >> 1) * kPairRows * kPairRows + (size_t)h * (kp * kPairRows + kp);
  float* Ttp = Tp + (size_t)nb * kPairRows * kPairRows;
  {
    // the factor goes out with agent-scope stores (written through to where any compute unit's agent-scope load
    // finds it), its transpose with ordinary ones; once every thread's stores are acknowledged the block is announced
    const BufferDesc tdesc = make_buffer(Tp, (size_t)(kp * kPairRows) * sizeof(float));
    for (int idx = tid; idx < kp * kp; idx += 512) {
      const int j = idx / kp, l = idx % kp;
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(Ms[j * LDM + l]), tdesc, (unsigned)(j * kPairRows + l) * 4u, 0, 16);
      Ttp[j * kPairRows + l] = Ms[l * LDM + j];
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) {
    const BufferDesc rdesc = make_buffer(reinterpret_cast<const float*>(ready + i), 8);
    const u32x2 w = {(unsigned)launch_id, (unsigned)(launch_id >> 32)};
    __builtin_amdgcn_raw_buffer_store_b64(w, rdesc, 0u, 0, 16);
  }
}

static size_t t_build_lds(int kp) {
  return sizeof(float) * ((size_t)kp * (kp + 4) + (size_t)invert_scratch_floats(kp));
}

}  // namespace fasth
