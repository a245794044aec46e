// Algorithm 1 Step 1: the k x k block factors T_i (factor_fused_kernel: a workgroup per block; team_factor_kernel:
// the Gram product of a block split over several workgroups).
// Included by fasth.hip, the library's single translation unit.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// The hand-off area of the workspace (words that workgroups of a later chain launch pass to each other, with the
// counters their tags continue from) starts every product at zero: whichever kernel builds the factors clears it,
// all its workgroups taking a share.
__device__ __forceinline__ void clear_exchange_area(unsigned* xch, unsigned words, unsigned wg, unsigned wgs) {
  // the area is 256-byte aligned and a whole number of 16-byte pieces
  u32x4* x4 = reinterpret_cast<u32x4*>(xch);
  for (unsigned w = wg * blockDim.x + threadIdx.x; w < words / 4u; w += wgs * blockDim.x) x4[w] = u32x4{0u, 0u, 0u, 0u};
}

// ------------------------------------------------------------------------------------------
// T_i = (diag(S)/2 + striu(S))^-1 from the Gram matrix S = V_i V_i^T (only the 16x16 tiles on or above the
// diagonal are formed): 16x16 diagonal blocks by unrolled back substitution, then [[T11, -T11 M12 T22], [0, T22]]
// doubles the block size each level with matrix-core products. Rows/columns >= k (padding) form an identity.
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

// ------------------------------------------------------------------------------------------
// Algorithm 1 Step 1 for blocks of 64 or 128 rows in one launch: the Gram product of a block is split over d among
// `split` workgroups (grid (split, nb), 8 kp threads; a workgroup stages 128-column slabs of its share in LDS and
// forms the upper tiles on the matrix cores), and the block's first workgroup, the leader, adds the partial
// matrices and inverts. What the others owe the leader is their partial matrix: they write it
// with agent-scope stores (written through to where any compute unit's agent-scope load finds it), wait until the
// stores are acknowledged and set an 8-byte "ready" word to a number the host draws anew for every launch; the
// leader polls the block's words, reads the partial matrices with agent-scope loads and clears the words, so a
// captured launch replayed with the same number starts from cleared words. (A workspace that has never been used
// holds arbitrary words: the chance that one equals the launch's 64-bit number is 2^-64.) The leader has the lowest
// index of its block's workgroups and those follow it directly, so they run (or have run) whenever it waits, also
// when the launch has more workgroups than the GPU has compute units. The wait is bounded like every wait between
// workgroups in this library: after wait_limit polls the leader raises the status word and goes on with what is
// there. (As two launches, partial matrices then sum and inverse, the same work took 18.3 us against 14.3 us at
// d = n = 1024, k = 64, and 39.8 against 35.2 us at d = n = 2048, k = 128.)
// Blocks of 32 rows that the team chain kernel applies in pairs are factored here as blocks of 64: by Lemma 1 the
// product of two consecutive blocks is a WY block of 64 rows whose factor is the inverse of the 64 x 64 matrix
// diag(S)/2 + striu(S), [[T1, -T1 S12 T2], [0, T2]] with the two blocks' own factors on its diagonal.
// For the chain kernel that applies two blocks of 64 rows per step the same launch forms, per pair of consecutive
// blocks a, b, the product of their rows S = V_a V_b^T (the S12 of Lemma 1, which that kernel applies between the two
// factors instead of a merged factor of 128 rows): npair more rows of workgroups, first in the grid, which stage the
// rows of both blocks, form all tiles of their share of d and hand them to the pair's first workgroup as a block's
// workgroups do; no workgroup waits for a factor.
// The leader fetches every group of four entries it owns from up to 16 / (KP / 32) partial matrices at once, so the
// sum costs a trip to memory per eight (four) partial matrices, not one per group.
// ------------------------------------------------------------------------------------------
struct TeamFactorArgs {
  const float* V;              // [n][d]
  float* Spart;                // [nb][split][kp][kp] partial Gram matrices (upper tiles)
  float* T;                    // [2][nb][kp][kp]
  unsigned long long* ready;   // [nb][split]
  unsigned long long launch_id;
  int d, k, kp, split, wait_limit;
  unsigned* xch;               // hand-off area of the chain kernels, cleared here
  unsigned xch_words;
  // For chain_team_wide_kernel (kp = 64 only): npair > 0 adds, per pair p of consecutive blocks, the product
  // S_p = V_2p V_2p+1^T of their rows (workgroups blockIdx.y < npair, the blocks' behind them), and every matrix is stored in the order in
  // which that kernel's threads read it.
  float* S;                    // [npair][2][kp][kp]: S_p, then its transpose
  int nblocks, npair;
};
// Up to two products of the same shape (the two orthogonal factors of an SVD layer) per launch: blockIdx.z picks.
struct TeamFactorPair {
  TeamFactorArgs a[2];
};

template <int VEC, int KP>  // KP: padded rows of a block, 64 or 128; 8 KP threads
__global__ void __launch_bounds__(8 * KP) team_factor_kernel(TeamFactorPair pair) {
  extern __shared__ __align__(16) float smem[];
  const TeamFactorArgs& p = pair.a[blockIdx.z];
  const int LD = kGramChunk + 4;
  constexpr int kp = KP;
  const int d = p.d, k = p.k, split = p.split;
  const int i = blockIdx.y, s = blockIdx.x;
  const int tid = threadIdx.x, nthreads = blockDim.x, wave = tid >> 6, nwaves = nthreads >> 6, lane = tid & 63;
  clear_exchange_area(p.xch, p.xch_words, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
  // The first npair rows of the grid form a pair's product S = V_a V_b^T instead of a block's Gram matrix: the rows of
  // both blocks (2 kp consecutive rows of V) in LDS, all kp / 16 squared tiles. They come first because they fetch
  // twice as much and are the last to start otherwise, when the launch has more workgroups than run at once.
  const bool pair_job = KP == 64 && i < p.npair;
  const int bi = i - p.npair;  // a block's workgroups: the block
  {
    float* Vs = smem;  // [kp][LD], a pair's [2 kp][LD]
    const int chunk = ((d + split - 1) / split + 3) & ~3;
    const int xbeg = s * chunk;
    const int xend = min(d, xbeg + chunk);
    const int kt = kp / 16;
    const int ntiles = pair_job ? kt * kt : kt * (kt + 1) / 2;
    constexpr int kMaxTilesPerWave = 3;  // kp = 128: 36 upper tiles over 16 waves; kp = 64: 10 over 8, a pair's 16 over 8
    f32x4 acc[kMaxTilesPerWave];
#pragma unroll
    for (int w = 0; w < kMaxTilesPerWave; ++w) acc[w] = f32x4{0.f, 0.f, 0.f, 0.f};
    // the block's k rows as one buffer: rows k .. kp - 1 of the padded block lie beyond it and read as zero
    const BufferDesc vdesc = pair_job ? make_buffer(p.V + (size_t)i * 2 * kp * d, (size_t)2 * kp * d * sizeof(float))
                                      : make_buffer(p.V + (size_t)bi * k * d, (size_t)k * d * sizeof(float));
    constexpr int XV = kGramChunk / VEC;  // loads per slab row
    constexpr int PER1 = 16 / VEC;        // loads per thread and slab: kp XV / nthreads with nthreads = 8 kp
    constexpr int PER = KP == 64 ? 2 * PER1 : PER1;  // room for a pair's rows; a block's workgroups use the first half
    const int nper = pair_job ? PER : PER1;
    // a slab is fetched while the one before it is multiplied
    BufVec<VEC> stage[PER];
    auto fetch_slab = [&](int x0) {
#pragma unroll
      for (int it = 0; it < PER; ++it) {
        const int idx = tid + it * nthreads, j = idx / XV, x = x0 + (idx % XV) * VEC;
        if (it < nper) stage[it] = buffer_load<VEC>(vdesc, x < xend ? (unsigned)(j * d + x) * 4u : kOob, 0);
      }
    };
    // tile t of this workgroup: (ti, tj) of the upper triangle, or of a pair's kt x kt tiles (rows of b behind those of a)
    auto tile_of = [&](int t, int& ti, int& tj) {
      if (pair_job) { ti = t / kt; tj = t % kt; return; }
      int rem = t;
      ti = 0;
      while (rem >= kt - ti) { rem -= kt - ti; ++ti; }
      tj = ti + rem;
    };
    fetch_slab(xbeg);
    for (int x0 = xbeg; x0 < xend; x0 += kGramChunk) {
#pragma unroll
      for (int it = 0; it < PER; ++it) {
        const int idx = tid + it * nthreads;
        if (it < nper) lds_store<VEC>(Vs + (idx / XV) * LD + (idx % XV) * VEC, stage[it]);
      }
      __syncthreads();
      if (x0 + kGramChunk < xend) fetch_slab(x0 + kGramChunk);
#pragma unroll
      for (int w = 0; w < kMaxTilesPerWave; ++w) {
        const int t = wave + nwaves * w;
        if (t < ntiles) {
          int ti, tj;
          tile_of(t, ti, tj);
          acc[w] = tile_mma<true>(Vs + ti * 16 * LD, LD, Vs + ((pair_job ? kp : 0) + tj * 16) * LD, LD, kGramChunk, acc[w]);
        }
      }
      __syncthreads();
    }
    // the partial matrix goes out with agent-scope stores
    const BufferDesc odesc = make_buffer(p.Spart + ((size_t)i * split + s) * kp * kp, (size_t)kp * kp * sizeof(float));
    const int li = lane & 15, q = lane >> 4;
#pragma unroll
    for (int w = 0; w < kMaxTilesPerWave; ++w) {
      const int t = wave + nwaves * w;
      if (t < ntiles) {
        int ti, tj;
        tile_of(t, ti, tj);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[w][jj]), odesc,
                                                (unsigned)((ti * 16 + 4 * q + jj) * kp + tj * 16 + li) * 4u, 0, 16);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  unsigned long long* ready = p.ready + (size_t)i * split;
  if (s != 0) {
    if (tid == 0) {
      const BufferDesc rdesc = make_buffer(reinterpret_cast<const float*>(ready + s), 8);
      const u32x2 w = {(unsigned)p.launch_id, (unsigned)(p.launch_id >> 32)};
      __builtin_amdgcn_raw_buffer_store_b64(w, rdesc, 0u, 0, 16);
    }
    return;
  }
  // the leader: wait for the other slices of the block
  if (wave == 0 && split > 1) {
    const BufferDesc rdesc = make_buffer(reinterpret_cast<const float*>(ready), (size_t)split * 8);
    const unsigned from = (unsigned)(lane >= 1 && lane < split ? lane : 1) * 8u;  // every lane reads some other slice's word
    bool gave_up = false;
    int polls = 0;
    for (;;) {
      const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rdesc, from, 0, 16);
      const unsigned long long v = ((unsigned long long)w.y << 32) | w.x;
      if (__all(v == p.launch_id)) break;
      if (polls++ >= p.wait_limit) { gave_up = true; break; }
      __builtin_amdgcn_s_sleep(2);
      asm volatile("" ::: "memory");
    }
    if (gave_up && lane == 0) __hip_atomic_store(&g_wait_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  const int LDM = kp + 4;
  float* Ms = smem;           // [kp][LDM]
  float* Xs = Ms + kp * LDM;  // scratch of the inversion
  {
    const BufferDesc sdesc = make_buffer(p.Spart + (size_t)i * split * kp * kp, (size_t)split * kp * kp * sizeof(float));
    // Four neighbouring entries of a row at a time (kp is a multiple of 16, so they share a 16 x 16 tile); tiles
    // below the diagonal hold nothing and are not read. All partial sums of an entry are in flight at once.
    // A trip to memory per batch of fetches: the 8 kp threads take kp / 32 groups of four entries each, and up to 16
    // fetches are in flight per thread (64 registers), i.e. all groups of a thread at once for up to 16 / (kp / 32)
    // partial matrices. The sum takes the partial matrices in their order whatever the batches.
    constexpr int NPOS = KP / 32;       // groups of four per thread
    constexpr int BATCH = 16 / NPOS;    // partial matrices per batch
    f32x4 sum[NPOS];
#pragma unroll
    for (int it = 0; it < NPOS; ++it) sum[it] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < split; s0 += BATCH) {
      f32x4 part[NPOS][BATCH];
#pragma unroll
      for (int it = 0; it < NPOS; ++it) {
        const int idx4 = tid + it * nthreads, j = idx4 / (kp / 4), l0 = (idx4 % (kp / 4)) * 4;
        const bool wanted = pair_job || (j / 16 <= l0 / 16 && j < k);
#pragma unroll
        for (int sb = 0; sb < BATCH; ++sb)
          part[it][sb] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                             sdesc, wanted && s0 + sb < split ? (unsigned)(((size_t)(s0 + sb) * kp * kp + 4 * (size_t)idx4) * 4u) : kOob, 0, 16));
      }
#pragma unroll
      for (int it = 0; it < NPOS; ++it) {
#pragma unroll
        for (int sb = 0; sb < BATCH; ++sb) sum[it] += part[it][sb];
      }
    }
#pragma unroll
    for (int it = 0; it < NPOS; ++it) {
      const int idx4 = tid + it * nthreads, j = idx4 / (kp / 4), l0 = (idx4 % (kp / 4)) * 4;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int l = l0 + u;
        float v = 0.f;
        if (pair_job) v = sum[it][u];
        else if (j < k && l < k && j <= l) v = j == l ? 0.5f * sum[it][u] : sum[it][u];
        else if (j == l) v = 1.f;
        Ms[j * LDM + l] = v;
      }
    }
  }
  __syncthreads();
  if (tid >= 1 && tid < split) ready[tid] = 0ull;  // the partial matrices are in: the words are cleared for the next launch
  // Order of a 64 x 64 matrix for chain_team_wide_kernel: its thread 16 g + c multiplies entries 4 c .. 4 c + 3 of rows
  // 2 g and 2 g + 1; those of row 2 g + e are the (512 e + 16 g + c)-th 16 bytes, so a wave's fetch of one e is 1 KiB in a row.
  auto chain_order_row = [](int idx) { return 2 * (((idx >> 2) & 511) >> 4) + (idx >> 11); };
  auto chain_order_col = [](int idx) { return 4 * ((idx >> 2) & 15) + (idx & 3); };
  if (pair_job) {
    float* Sp = p.S + (size_t)i * 2 * kp * kp;
    for (int idx = tid; idx < kp * kp; idx += nthreads) {
      const int j = chain_order_row(idx), l = chain_order_col(idx);
      Sp[idx] = Ms[j * LDM + l];
      Sp[kp * kp + idx] = Ms[l * LDM + j];
    }
    return;
  }
  diag_scratch_fill(Ms, Xs, kp, LDM);
  invert_upper_lds<KP == 64>(Ms, Xs, kp, LDM);  // 512 threads have the registers to fetch a diagonal block at once
  // T_i and, nb factors further on, its transpose: a chain kernel then reads rows of op(T_i) in either direction
  float* Ti = p.T + (size_t)bi * kp * kp;
  float* Tti = Ti + (size_t)p.nblocks * kp * kp;
  if (KP == 64 && p.npair > 0) {
    for (int idx = tid; idx < kp * kp; idx += nthreads) {
      const int j = chain_order_row(idx), l = chain_order_col(idx);
      Ti[idx] = Ms[j * LDM + l];
      Tti[idx] = Ms[l * LDM + j];
    }
    return;
  }
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

static size_t t_build_lds(int kp) {
  return sizeof(float) * ((size_t)kp * (kp + 4) + (size_t)invert_scratch_floats(kp));
}

}  // namespace fasth
