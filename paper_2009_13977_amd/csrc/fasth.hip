// FastH for CDNA4 (gfx950): kernels and the C ABI declared in include/fasth.h.
//
// Notation follows the paper (arXiv 2009.13977): d = vector length, n = number of reflections,
// m = mini-batch columns, k = block size (Section 3.3), nb = n / k blocks P_i (Eq. 2).
//
// Block form used here. For the k rows V_i of one block, with S = V_i V_i^T,
//   P_i = H_{(i-1)k+1} ... H_{ik} = I - V_i^T T_i V_i,   T_i = (diag(S)/2 + striu(S))^-1.
// This is the WY form of Lemma 1 (Y = V_i^T, W = V_i^T T_i / 2) kept as the k x k factor T_i, so
// Step 1 of Algorithm 1 is one Gram product per block (matrix cores) plus a k x k triangular
// inverse, and P_i^T = I - V_i^T T_i^T V_i needs no second factor.
//
// Kernels
//   gram_partial_kernel  Algorithm 1 Step 1a: partial Gram matrices of every block (MFMA)
//   t_build_kernel       Algorithm 1 Step 1b: T_i by blocked triangular inversion (MFMA)
//   factor_fused_kernel  Algorithm 1 Step 1 in one kernel for block sizes up to 32
//   chain_kernel         Algorithm 1 Step 2 / Algorithm 2 Step 1: the sequential block chain,
//                        one workgroup per column of X (columns are independent)
//   dv_kernel            Algorithm 2 Step 2 as dense products per block (MFMA)
//   seq_*                the one-reflection-at-a-time comparison
//   dsigma_kernel        the diagonal step of the SVD layer
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <type_traits>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "fasth.h"
#include "fasth_device.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// Host-side shape bookkeeping
// ------------------------------------------------------------------------------------------

constexpr int kMaxBlock = 128;     // largest k: a k x k factor must fit in LDS with scratch
constexpr int kMaxD = 16384;       // chain kernel: 1024 threads x 16 elements
constexpr int kGramChunk = 128;    // columns of V per LDS tile in the Gram kernel
constexpr int kMaxGramSplit = 16;  // partial Gram matrices per block
constexpr int kDvTile = 64;        // columns of dV per workgroup
constexpr int kDvMChunk = 32;      // mini-batch columns per LDS tile in the dV kernel

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int padded_block(int k) {
  int kp = 16;
  while (kp < k) kp *= 2;
  return kp;
}

struct Layout {
  int kp, nb, gram_split;
  size_t off_T, off_Spart, off_saveA, off_saveCa, off_saveG, off_saveCg, total;
};

static Layout make_layout(int d, int n, int m, int k) {
  Layout L;
  L.kp = padded_block(k);
  L.nb = n / k;
  int split = (d + kGramChunk - 1) / kGramChunk;
  L.gram_split = split > kMaxGramSplit ? kMaxGramSplit : split;
  size_t off = 256;  // header, reserved
  auto take = [&](size_t floats) {
    size_t o = off;
    off = align_up(off + floats * sizeof(float), 256);
    return o;
  };
  L.off_T = take((size_t)L.nb * L.kp * L.kp);
  L.off_Spart = take((size_t)L.nb * L.gram_split * L.kp * L.kp);
  L.off_saveA = take((size_t)L.nb * m * d);
  L.off_saveCa = take((size_t)m * n);
  L.off_saveG = take((size_t)L.nb * m * d);
  L.off_saveCg = take((size_t)m * n);
  L.total = off;
  return L;
}

static int check_shape(const fasth_shape* s) {
  if (!s) return FASTH_EINVAL;
  if (s->d < 1 || s->n < 1 || s->m < 1 || s->k < 1) return FASTH_EINVAL;
  if (s->n % s->k != 0) return FASTH_EINVAL;
  if (s->transpose != 0 && s->transpose != 1) return FASTH_EINVAL;
  if (s->k > kMaxBlock || s->d > kMaxD || s->m > 65535) return FASTH_EUNSUPPORTED;
  return FASTH_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define FASTH_HIP(call)                      \
  do {                                       \
    hipError_t e_ = (call);                  \
    if (e_ != hipSuccess) return FASTH_EHIP; \
  } while (0)

// Optional per-kernel timing for benchmarks: a pair of HIP events around every launch.
namespace prof {
struct Rec { int id; hipEvent_t beg, end; };
static bool enabled = false;
static std::vector<Rec> recs;
static std::vector<hipEvent_t> pool;
static hipEvent_t get_event() {
  if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
struct Scope {
  Rec r{-1, nullptr, nullptr};
  hipStream_t st;
  Scope(int id, hipStream_t s) : st(s) {
    if (!enabled) return;
    r.id = id; r.beg = get_event(); r.end = get_event();
    if (r.beg) (void)hipEventRecord(r.beg, st);
  }
  ~Scope() {
    if (r.id < 0) return;
    if (r.end) (void)hipEventRecord(r.end, st);
    recs.push_back(r);
  }
};
}  // namespace prof

template <typename K>
static int allow_lds(K kernel, size_t bytes) {
  if (bytes > 64 * 1024) {
    FASTH_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  }
  return FASTH_OK;
}

// ------------------------------------------------------------------------------------------
// Algorithm 1 Step 1a: partial Gram matrices S_i = V_i V_i^T, split over d.
// grid (gram_split, nb), 256 threads. Only the 16x16 tiles on or above the diagonal are formed.
// ------------------------------------------------------------------------------------------

template <int VEC>  // VEC = 4 when d is a multiple of 4 (16-byte loads), else 1
__global__ void __launch_bounds__(256) gram_partial_kernel(const float* __restrict__ V, float* __restrict__ Spart,
                                                           int d, int k, int kp, int gram_split) {
  extern __shared__ __align__(16) float smem[];
  const int LD = kGramChunk + 4;
  float* Vs = smem;  // [kp][LD]
  const int i = blockIdx.y, s = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
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
        acc[w] = tile_mma(Vs + ti * 16 * LD, LD, 1, Vs + tj * 16 * LD, 1, LD, kGramChunk, acc[w]);
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

// In-place inverse of the upper-triangular kp x kp matrix Ms (row stride LDM) in LDS by block
// doubling; Xs is scratch of max(kp * (kp/2 + 4) / 2 + 64, kp * 17) floats. Called by every thread of the workgroup
// (a multiple of 64 threads); Ms must be complete (barrier) on entry and is complete on return.
__device__ __forceinline__ void invert_upper_lds(float* Ms, float* Xs, int kp, int LDM) {
  const int tid = threadIdx.x, nthreads = blockDim.x, wave = tid >> 6, nwaves = nthreads >> 6, lane = tid & 63;
  // 16x16 diagonal blocks: thread c of a block solves for column c by back substitution, fully
  // unrolled so that the reads of M (a copy in Xs) are independent of the values being computed.
  float* Ds = Xs;  // [kp/16][16][17]
  if (tid < kp) {
    const int base = tid & ~15, c = tid & 15;
#pragma unroll
    for (int r = 0; r < 16; ++r) Ds[(base + r) * 17 + c] = Ms[(base + r) * LDM + base + c];
  }
  __syncthreads();
  if (tid < kp) {
    const int base = tid & ~15, c = tid & 15;
    const float* D = Ds + base * 17;
    float x[16], rdiag[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) rdiag[r] = 1.f / D[r * 17 + r];  // all sixteen at once, off the dependent chain
#pragma unroll
    for (int r = 15; r >= 0; --r) {
      float sum = r == c ? 1.f : 0.f;
      // oldest x first: the value computed last enters last, so each row adds one multiply-add to the chain
#pragma unroll
      for (int l = 15; l > r; --l) sum = fmaf(-D[r * 17 + l], x[l], sum);
      x[r] = sum * rdiag[r];  // rows below c stay exactly zero
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) Ms[(base + r) * LDM + base + c] = x[r];
  }
  __syncthreads();
  const int li = lane & 15, q = lane >> 4;
  for (int b = 16; b < kp; b *= 2) {
    const int tpb = b / 16, per_pair = tpb * tpb, items = (kp / (2 * b)) * per_pair;
    const int LDX = b + 4;
    for (int it = wave; it < items; it += nwaves) {  // X = M12 T22
      const int pr = it / per_pair, ti = (it % per_pair) / tpb, tj = it % tpb, r0 = pr * 2 * b;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = tile_mma(Ms + (r0 + 16 * ti) * LDM + r0 + b, LDM, 1, Ms + (r0 + b) * LDM + r0 + b + 16 * tj, LDM, 1, b, acc);
      float* X = Xs + pr * b * LDX;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) X[(16 * ti + 4 * q + jj) * LDX + 16 * tj + li] = acc[jj];
    }
    __syncthreads();
    for (int it = wave; it < items; it += nwaves) {  // T12 = -T11 X
      const int pr = it / per_pair, ti = (it % per_pair) / tpb, tj = it % tpb, r0 = pr * 2 * b;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      acc = tile_mma(Ms + (r0 + 16 * ti) * LDM + r0, LDM, 1, Xs + pr * b * LDX + 16 * tj, LDX, 1, b, acc);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) Ms[(r0 + 16 * ti + 4 * q + jj) * LDM + r0 + b + 16 * tj + li] = -acc[jj];
    }
    __syncthreads();
  }
}

__global__ void __launch_bounds__(1024) t_build_kernel(const float* __restrict__ Spart, float* __restrict__ T,
                                                      int k, int kp, int gram_split) {
  extern __shared__ float smem[];
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
  invert_upper_lds(Ms, Xs, kp, LDM);
  float* Ti = T + (size_t)i * kp * kp;
  for (int idx = tid; idx < kp * kp; idx += nthreads) Ti[idx] = Ms[(idx / kp) * LDM + idx % kp];
}

// Algorithm 1 Step 1 in one kernel for small blocks (kp = 16 KT <= 32): one workgroup of 8 waves per
// block streams the block's rows through LDS in 128-column slabs; wave w multiplies columns
// [16 w, 16 w + 16) of each slab, the 8 partial Gram matrices are added through LDS, and the same
// workgroup inverts. Saves a launch and the round trip of the partial sums through memory.
// Up to two products (the two orthogonal factors of an SVD layer) are factored by one launch:
// blockIdx.y picks the product, blockIdx.x its block.
struct FactorPair {
  const float* V[2];  // [n][d]
  float* T[2];        // [nb][kp][kp]
  int d[2], k[2], nb[2];
};

template <int KT, int VEC>  // VEC = 4 when d is a multiple of 4 (16-byte loads), else 1
__global__ void __launch_bounds__(512) factor_fused_kernel(FactorPair fp) {
  const int which = blockIdx.y;
  if ((int)blockIdx.x >= fp.nb[which]) return;  // whole workgroup, before any barrier
  const float* __restrict__ V = fp.V[which];
  float* __restrict__ T = fp.T[which];
  const int d = fp.d[which], k = fp.k[which];
  constexpr int kp = 16 * KT, LD = kGramChunk + 4, NTILE = KT * (KT + 1) / 2, NW = 8, LDM = kp + 4;
  constexpr int PER = kp * kGramChunk / 512 / VEC;  // loads per thread and slab
  constexpr int XV = kGramChunk / VEC;              // loads per slab row
  __shared__ __align__(16) float Vs[kp * LD];
  __shared__ float Red[NW * NTILE * 256];
  __shared__ float Ms[kp * LDM];
  __shared__ float Xs[(kp * (kp / 2 + 4) / 2 + 64) > kp * 17 ? (kp * (kp / 2 + 4) / 2 + 64) : kp * 17];
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
        __syncthreads();
      }
    }
  }
#pragma unroll
  for (int t = 0; t < NTILE; ++t) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) Red[(wave * NTILE + t) * 256 + (4 * q + jj) * 16 + li] = acc[t][jj];
  }
  __syncthreads();
  for (int idx = tid; idx < kp * kp; idx += 512) {
    const int j = idx / kp, l = idx % kp;
    float v = 0.f;
    if (j < k && l < k && j <= l) {
      const int ti = j / 16, tj = l / 16;
      const int t = ti * KT - ti * (ti - 1) / 2 + (tj - ti);  // index of tile (ti, tj) in the upper-triangle order
#pragma unroll
      for (int w = 0; w < NW; ++w) v += Red[(w * NTILE + t) * 256 + (j % 16) * 16 + l % 16];
      if (j == l) v *= 0.5f;
    } else if (j == l) {
      v = 1.f;
    }
    Ms[j * LDM + l] = v;
  }
  __syncthreads();
  invert_upper_lds(Ms, Xs, kp, LDM);
  float* Ti = T + (size_t)i * kp * kp;
  for (int idx = tid; idx < kp * kp; idx += 512) Ti[idx] = Ms[(idx / kp) * LDM + idx % kp];
}

static size_t t_build_lds(int kp) {
  size_t scratch = (size_t)kp * (kp / 2 + 4) / 2 + 64;
  if (scratch < (size_t)kp * 17) scratch = (size_t)kp * 17;
  return sizeof(float) * ((size_t)kp * (kp + 4) + scratch);
}

// ------------------------------------------------------------------------------------------
// The sequential block chain (Algorithm 1 Step 2; Algorithm 2 Step 1, Eq. 3).
// One workgroup per column of the d x m input: columns never interact, so no workgroup waits for
// another. Per block i:  B = V_i a,  C = op(T_i) B,  a <- a - V_i^T C,
// op(T) = T for P_i (blocks nb..1), T^T for P_i^T (blocks 1..nb).
// Thread t owns elements x = t + u * blockDim.x of the column. The k inner products of a block are
// independent, which is the parallelism FastH adds over the one-at-a-time algorithm.
// Saved for the backward pass: the input column of every block and the coefficient vector C.
// ------------------------------------------------------------------------------------------

// Diagonal factor applied to row x of a chain's input (Section 2.2 and Table 1):
// 1: sigma, 2: 1/sigma (inverse), 3: e^sigma (matrix exponential), 4: (1 - sigma)/(1 + sigma) (Cayley map).
__device__ __forceinline__ float diag_factor(int mode, float sigma) {
  switch (mode) {
    case 1: return sigma;
    case 2: return 1.f / sigma;
    case 3: return expf(sigma);
    case 4: return (1.f - sigma) / (1.f + sigma);
    default: return 1.f;
  }
}

struct ChainArgs {
  const float* V;         // [n][d]
  const float* T;         // [nb][kp][kp]
  const float* in;        // [d][m]
  float* out;             // [d][m]
  float* save_in;         // [nb][m][d] or null
  float* save_c;          // [m][n] or null
  const float* in_scale;  // [d] or null: input row x is multiplied by diag_factor(in_scale_mode, in_scale[x])
  int in_scale_mode;
  int in_rows;            // rows of `in` that exist; rows in_rows..d-1 of the chain's input are zero
  int d, n, m, k, kp, nb;
  int transpose;
  int sub;                // chain_pipe_kernel: steps per block (set by its launcher)
  // Optional side product of the SVD layers' backward pass, which has the chain's input as one operand:
  // ds_out[r] = s'(in_scale[r]) sum_l in[r][l] ds_z1[r][l] for r < ds_rows (s = diag_factor(in_scale_mode, .)).
  // Null ds_out: not wanted. Kernels that cannot take it along leave it to a launch of dsigma_kernel.
  const float* ds_z1;     // [ds_rows][m]
  float* ds_out;          // [ds_rows]
  int ds_rows;
};

// Gradient of the diagonal step of the SVD layer (Section 2.2), one wave per row: with Z2 = s * Z1 row-wise
// (s = sigma, 1/sigma or a function of sigma),
//   ds_r = sum_l dZ2[r][l] Z1[r][l];  dsigma_r = ds_r * s'(sigma_r)  (e.g. -ds_r / sigma_r^2 for s = 1/sigma).
__device__ __forceinline__ void dsigma_row(const float* __restrict__ dZ2, const float* __restrict__ Z1,
                                           const float* __restrict__ sigma, float* __restrict__ dsigma, int row,
                                           int m, int mode) {
  const int lane = threadIdx.x & 63;
  float r[1] = {0.f};
  for (int l = lane; l < m; l += 64) r[0] += dZ2[(size_t)row * m + l] * Z1[(size_t)row * m + l];
  wave_reduce_multi<1>(r);
  if (lane == 0) {
    // chain rule from the diagonal factor s(sigma) to sigma: mode = diag_factor mode
    float v = r[0];
    const float sg = sigma[row];
    if (mode == 2) v = -v / (sg * sg);
    else if (mode == 3) v *= expf(sg);
    else if (mode == 4) v *= -2.f / ((1.f + sg) * (1.f + sg));
    dsigma[row] = v;
  }
}

__global__ void __launch_bounds__(256) dsigma_kernel(const float* __restrict__ dZ2, const float* __restrict__ Z1,
                                                     const float* __restrict__ sigma, float* __restrict__ dsigma,
                                                     int d, int m, int mode) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row < d) dsigma_row(dZ2, Z1, sigma, dsigma, row, m, mode);
}

template <int U>
__global__ void __launch_bounds__(1024) chain_kernel(ChainArgs p) {
  extern __shared__ float smem[];
  const int nthreads = blockDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const int col = blockIdx.x;
  const int d = p.d, k = p.k, kp = p.kp, m = p.m;
  const int LDT = kp + 1;
  float* Ts = smem;               // [kp][LDT]
  float* Bpart = Ts + kp * LDT;   // [nw][kp]
  float* Bv = Bpart + nw * kp;    // [kp]
  float* Cv = Bv + kp;            // [kp]
  float a[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int x = tid + u * nthreads;
    float v = 0.f;
    if (x < d && x < p.in_rows) {
      v = p.in[(size_t)x * m + col];
      if (p.in_scale_mode) v *= diag_factor(p.in_scale_mode, p.in_scale[x]);
    }
    a[u] = v;
  }
  const int sel = reduce_sel<8>(lane);
  for (int s = 0; s < p.nb; ++s) {
    const int i = p.transpose ? s : p.nb - 1 - s;
    const float* Vi = p.V + (size_t)i * k * d;
    const float* Ti = p.T + (size_t)i * kp * kp;
    for (int idx = tid; idx < kp * kp; idx += nthreads) Ts[(idx / kp) * LDT + idx % kp] = Ti[idx];
    if (p.save_in) {
      float* dst = p.save_in + ((size_t)i * m + col) * d;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int x = tid + u * nthreads;
        if (x < d) dst[x] = a[u];
      }
    }
    for (int j0 = 0; j0 < k; j0 += 8) {
      float pj[8];
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        pj[jj] = 0.f;
        if (j0 + jj < k) {
          const float* vr = Vi + (size_t)(j0 + jj) * d;
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int x = tid + u * nthreads;
            if (x < d) pj[jj] += vr[x] * a[u];
          }
        }
      }
      wave_reduce_multi<8>(pj);
      if ((lane & reduce_writer_mask<8>()) == 0) Bpart[wave * kp + j0 + sel] = pj[0];
    }
    __syncthreads();
    if (tid < kp) {
      float b = 0.f;
      if (tid < k)
        for (int w = 0; w < nw; ++w) b += Bpart[w * kp + tid];
      Bv[tid] = b;
    }
    __syncthreads();
    if (tid < kp) {
      float c = 0.f;
      if (p.transpose) {
        for (int l = 0; l < kp; ++l) c += Ts[l * LDT + tid] * Bv[l];
      } else {
        for (int l = 0; l < kp; ++l) c += Ts[tid * LDT + l] * Bv[l];
      }
      Cv[tid] = c;
      if (p.save_c && tid < k) p.save_c[(size_t)col * p.n + i * k + tid] = c;
    }
    __syncthreads();
    for (int j = 0; j < k; ++j) {
      const float c = Cv[j];
      const float* vr = Vi + (size_t)j * d;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int x = tid + u * nthreads;
        if (x < d) a[u] -= c * vr[x];
      }
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int x = tid + u * nthreads;
    if (x < d) p.out[(size_t)x * m + col] = a[u];
  }
}

// ---- Register-resident chain kernels -------------------------------------------------------
// Thread t owns one VW-wide chunk of the column (x = VW t .. VW t + VW - 1), so a wave load of one
// row of V covers 64 VW contiguous floats and the whole k x d block V_i is K * VW registers per
// thread. V_i is read from memory once per block and used for both products.
//
// Two register copies: the rows of block i+1 are loaded a couple at a time between the multiply-adds
// of block i (during B = V_i a, during the reduction and during a -= V_i^T C), which feeds the CU's
// address unit (64 B per clock) evenly instead of in one burst that stalls the wave behind it.
// Blocks too large for two copies are applied as steps of fewer rows (SUB below).
// The barriers order LDS traffic only, so global loads stay in flight across them.
template <int VW> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef float2 type; };
template <> struct VecOf<4> { typedef float4 type; };

template <int VW>
struct Chunk {
  float e[VW];
};

template <int VW>
__device__ __forceinline__ Chunk<VW> load_chunk(const float* ptr) {
  Chunk<VW> c;
  const typename VecOf<VW>::type v = *reinterpret_cast<const typename VecOf<VW>::type*>(ptr);
  if constexpr (VW == 1) { c.e[0] = v; }
  else if constexpr (VW == 2) { c.e[0] = v.x; c.e[1] = v.y; }
  else { c.e[0] = v.x; c.e[1] = v.y; c.e[2] = v.z; c.e[3] = v.w; }
  return c;
}

template <int VW>
__device__ __forceinline__ void store_chunk(float* ptr, const Chunk<VW>& c) {
  typename VecOf<VW>::type v;
  if constexpr (VW == 1) { v = c.e[0]; }
  else if constexpr (VW == 2) { v.x = c.e[0]; v.y = c.e[1]; }
  else { v.x = c.e[0]; v.y = c.e[1]; v.z = c.e[2]; v.w = c.e[3]; }
  *reinterpret_cast<typename VecOf<VW>::type*>(ptr) = v;
}

// Loads this thread's part of column `col` of a [d][m] matrix, with the optional row scaling.
template <int VW>
__device__ __forceinline__ Chunk<VW> load_column_chunk(const ChainArgs& p, int col, unsigned x0, bool ok) {
  Chunk<VW> a;
#pragma unroll
  for (int r = 0; r < VW; ++r) {
    float v = 0.f;
    if (ok && x0 + r < (unsigned)p.in_rows) {
      v = p.in[(size_t)(x0 + r) * p.m + col];
      if (p.in_scale_mode) v *= diag_factor(p.in_scale_mode, p.in_scale[x0 + r]);
    }
    a.e[r] = v;
  }
  return a;
}

template <int K, int VW, int NT>
struct PipeRegs {
  static constexpr int G0 = (NT / K) < 16 ? (NT / K) : 16;
  static constexpr int G = G0 < K ? G0 : K;  // threads sharing one row of T
  static constexpr int LPT = K / G;
  Chunk<VW> v[K];
  float t[LPT];
};

// A block of more than K rows is applied as several steps of K rows. The diagonal K x K blocks of its factor T_i
// are the factors of the row groups (T_i is triangular and the groups are consecutive reflections), the
// coefficients of the steps put together are T_i V_i a, and the block's input is saved at its first step,
// so nothing downstream sees the difference; p.nb counts the steps. SUB is the number of steps per block
// (0: taken from p.sub at run time). PAD: k is not a multiple of K, so a block's last step has fewer than K
// rows; the missing rows repeat the last one and their inner products and coefficients are forced to zero.
// RL: rows of the next block fetched during the reduction; P1: during the first product (0: half of the rest).
template <int K, int VW, int NT, int RL = 0, int SUB = 1, bool PAD = false, int P1 = 0>
__global__ void __launch_bounds__(NT) chain_pipe_kernel(ChainArgs p) {
  typedef PipeRegs<K, VW, NT> Regs;
  constexpr int NW = NT / 64, G = Regs::G, LPT = Regs::LPT;
  constexpr int PR = P1 > 0 ? P1 : (K - RL) / 2;  // rows of the next block fetched during the first product
  constexpr int PR2 = K - RL - PR;                  // ... and during the second
  constexpr int S1 = K / PR, S2 = K / PR2;          // one fetch every S1 (S2) rows of the product
  static_assert(PR >= 1 && PR2 >= 1 && S1 >= 1 && S2 >= 1, "prefetch split");
  static_assert(K % 4 == 0 && K * G <= NT && LPT >= 1, "shape");
  static_assert(RL % 2 == 0 && RL <= K / 4 && (RL == 0 || K >= 8), "prefetch split");
  static_assert(!PAD || SUB == 0, "ragged steps take the step count at run time");
  __shared__ __align__(16) float Bpart[NW][K];
  __shared__ __align__(16) float Cv[K];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = blockIdx.x, m = p.m, d = p.d;
  if (col >= m) {  // workgroups beyond the columns: the side product, on compute units the chain leaves idle
    const int row = (col - m) * NW + wave;
    if (row < p.ds_rows) dsigma_row(p.in, p.ds_z1, p.in_scale, p.ds_out, row, m, p.in_scale_mode);
    return;
  }
  const int trow = tid / G, tg = tid % G;
  const bool t_active = tid < K * G;
  const int nb = p.nb;
  // A wave whose chunks all lie beyond d and that has no row of T to multiply only keeps the barrier count:
  // it issues no loads, which would cost the compute unit's address unit as much as useful ones.
  if (wave * 64 * VW >= d && wave * 64 >= K * G) {
    if (lane < K) Bpart[wave][lane] = 0.f;
    for (int s = 0; s < nb; ++s) {
      lds_barrier();
      lds_barrier();
    }
    return;
  }
  // Threads whose chunk lies beyond d read chunk 0 (always valid memory) and keep their part of
  // the column at zero, so they contribute nothing and need no branch per load.
  const bool ok = VW * tid < d;
  const unsigned x0 = ok ? VW * tid : 0;
  Chunk<VW> a = load_column_chunk<VW>(p, col, x0, ok);
  const int sel = reduce_sel<K>(lane);
  auto block_of = [&](int s) { return p.transpose ? s : nb - 1 - s; };
  const int sub = SUB > 0 ? SUB : p.sub;
  auto step_block = [&](int i) { return SUB == 1 ? i : i / sub; };
  auto step_part = [&](int i) { return SUB == 1 ? 0 : i % sub; };
  auto rows_valid = [&](int i) { return PAD ? min(K, p.k - step_part(i) * K) : K; };
  // uniform row base (scalar registers) + 32-bit per-lane offset
  auto row_ptr = [&](int i, int j) {
    if constexpr (PAD) {
      const int row = step_block(i) * p.k + step_part(i) * K + min(j, rows_valid(i) - 1);
      return p.V + (size_t)row * (size_t)d + x0;
    } else {
      return p.V + ((size_t)i * K + j) * (size_t)d + x0;
    }
  };
  auto load_t = [&](int i, Regs& r) {
    const int LDT = (SUB > 0 && K * SUB >= 16) ? K * SUB : p.kp;  // row stride of the stored factor
    const float* Ti = p.T + (size_t)step_block(i) * LDT * LDT + (size_t)step_part(i) * (K * LDT + K);
    const int row = t_active ? trow : 0;
#pragma unroll
    for (int e = 0; e < LPT; ++e) {
      const int l = tg * LPT + e;  // a thread's columns are consecutive: its partial sums come as 16-byte LDS reads
      r.t[e] = p.transpose ? Ti[l * LDT + row] : Ti[row * LDT + l];
    }
  };

  // Applies block i held in `cur` while fetching block inext into `nxt`.
  auto apply_block = [&](int i, Regs& cur, int inext, Regs& nxt) {
    if (p.save_in && ok && (SUB == 1 || step_part(i) == (p.transpose ? 0 : sub - 1)))
      store_chunk<VW>(p.save_in + ((size_t)step_block(i) * m + col) * d + x0, a);
    const int kv = rows_valid(i);
    float pj[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
      if (j % S1 == 0 && j / S1 < PR) {
        nxt.v[j / S1] = load_chunk<VW>(row_ptr(inext, j / S1));
        __builtin_amdgcn_sched_barrier(0);
      }
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < VW; ++r) acc = fmaf(cur.v[j].e[r], a.e[r], acc);
      pj[j] = (PAD && j >= kv) ? 0.f : acc;
    }
    load_t(inext, nxt);
    if constexpr (RL > 0) {
      auto prefetch = [&](int t) {
        if (t % 4 == 0 && t / 4 < RL) {
          __builtin_amdgcn_sched_barrier(0);
          nxt.v[PR + t / 4] = load_chunk<VW>(row_ptr(inext, PR + t / 4));
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      wave_reduce_multi_reg<K>(pj, prefetch);
    } else {
      wave_reduce_multi_reg<K>(pj);
    }
    if ((lane & reduce_writer_mask<K>()) == 0) Bpart[wave][sel] = pj[0];
    lds_barrier();
    if (t_active) {
      float c = 0.f;
      if constexpr (LPT % 4 == 0) {
#pragma unroll
        for (int e4 = 0; e4 < LPT / 4; ++e4) {
          float4 b = *reinterpret_cast<const float4*>(&Bpart[0][tg * LPT + 4 * e4]);
#pragma unroll
          for (int w = 1; w < NW; ++w) {
            const float4 t4 = *reinterpret_cast<const float4*>(&Bpart[w][tg * LPT + 4 * e4]);
            b.x += t4.x; b.y += t4.y; b.z += t4.z; b.w += t4.w;
          }
          c = fmaf(cur.t[4 * e4], b.x, c);
          c = fmaf(cur.t[4 * e4 + 1], b.y, c);
          c = fmaf(cur.t[4 * e4 + 2], b.z, c);
          c = fmaf(cur.t[4 * e4 + 3], b.w, c);
        }
      } else {
#pragma unroll
        for (int e = 0; e < LPT; ++e) {
          const int l = tg * LPT + e;
          float b = Bpart[0][l];
#pragma unroll
          for (int w = 1; w < NW; ++w) b += Bpart[w][l];
          c = fmaf(cur.t[e], b, c);
        }
      }
      c = group_sum<G>(c);
      if (PAD && trow >= kv) c = 0.f;
      if (tg == 0) {
        Cv[trow] = c;
        if constexpr (PAD) {
          if (p.save_c && trow < kv) p.save_c[(size_t)col * p.n + (size_t)step_block(i) * p.k + step_part(i) * K + trow] = c;
        } else {
          if (p.save_c) p.save_c[(size_t)col * p.n + (size_t)i * K + trow] = c;
        }
      }
    }
    lds_barrier();
    // The coefficient vector comes from LDS eight values at a time, one group ahead of its use: holding all K
    // would push more of the second register copy into the accumulator file (115.7 -> 114.3 us at the headline).
    constexpr int CG = K >= 16 ? 8 : K;
    float cc[2][CG];
    auto read_cc = [&](int grp, float (&dst)[CG]) {
#pragma unroll
      for (int j4 = 0; j4 < CG / 4; ++j4) {
        const float4 c4 = reinterpret_cast<const float4*>(Cv)[grp * (CG / 4) + j4];
        dst[4 * j4] = c4.x; dst[4 * j4 + 1] = c4.y; dst[4 * j4 + 2] = c4.z; dst[4 * j4 + 3] = c4.w;
      }
    };
    read_cc(0, cc[0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < K; ++j) {
      if (j % CG == 0 && j + CG < K) {
        read_cc(j / CG + 1, cc[(j / CG + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (j % S2 == 0 && j / S2 < PR2) {
        nxt.v[PR + RL + j / S2] = load_chunk<VW>(row_ptr(inext, PR + RL + j / S2));
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int r = 0; r < VW; ++r) a.e[r] = fmaf(-cc[(j / CG) & 1][j % CG], cur.v[j].e[r], a.e[r]);
    }
    if (!ok) {
#pragma unroll
      for (int r = 0; r < VW; ++r) a.e[r] = 0.f;
    }
  };

  Regs ra, rb;
#pragma unroll
  for (int j = 0; j < K; ++j) ra.v[j] = load_chunk<VW>(row_ptr(block_of(0), j));
  load_t(block_of(0), ra);
  int s = 0;
  for (; s + 1 < nb; s += 2) {
    apply_block(block_of(s), ra, block_of(s + 1), rb);
    apply_block(block_of(s + 1), rb, block_of(s + 2 < nb ? s + 2 : s + 1), ra);
  }
  if (s < nb) apply_block(block_of(s), ra, block_of(s), rb);
  if (ok) {
#pragma unroll
    for (int r = 0; r < VW; ++r) p.out[(size_t)(x0 + r) * m + col] = a.e[r];
  }
}

template <int K, int VW, int NT, int RL = 0, int SUB = 1, bool PAD = false, int P1 = 0>
static int launch_chain_pipe(const ChainArgs& args, hipStream_t stream) {
  ChainArgs a = args;
  a.sub = SUB > 0 ? SUB : (args.k + K - 1) / K;
  a.nb = args.nb * a.sub;
  if ((size_t)VW * NT < (size_t)a.d || (PAD ? a.sub * K > a.kp : a.sub * K != a.k)) return FASTH_EINVAL;
  const int side = a.ds_out ? (a.ds_rows + NT / 64 - 1) / (NT / 64) : 0;
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream);
  hipLaunchKernelGGL((chain_pipe_kernel<K, VW, NT, RL, SUB, PAD, P1>), dim3(a.m + side), dim3(NT), 0, stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

// ---- Matrix-core chain kernel for wide mini-batches ------------------------------------------
// With many columns the two products of a block step, B = V_i A and A -= V_i^T C, are dense contractions with a
// real N dimension, so they go to the fp32 matrix cores: one workgroup of 4 (d <= 1024) or 8 waves per tile of 16 columns.
//  * The d x 16 tile of A lives in the accumulator registers for the whole chain. The x axis is cut into groups
//    of 64; wave w of NW owns groups w, w + NW, ... Within a group, accumulator tile r (0..3), register j of lane
//    (q, i) = (lane / 16, lane % 16) holds A(x = 64 g + 16 q + 4 j + r, column i): the order in which a
//    contraction runs over x is free, and this one lets the same registers serve as the product's output tile
//    (A -= V^T C) and as the B operand of the next step's first product without any shuffle, while every fetch
//    of V from LDS is 16 bytes wide.
//  * Rows are taken 16 at a time (a block of more rows in several steps with the diagonal 16 x 16 blocks of its
//    factor, as in chain_pipe_kernel). Each wave stages only its own groups of the 16 rows in LDS (fetched
//    from memory into registers a step ahead with row-contiguous 16-byte loads, written to LDS when the step's
//    second product has read the old rows); both products read them. 75 KiB of LDS and under 256 registers per
//    workgroup let two workgroups share a compute unit and fill each other's waits.
//  * One barrier per step: the waves' partial B (16 x 16 each) meet in LDS, then every wave forms
//    C = op(T) B itself (4 matrix instructions), which is already laid out as the B operand of the update.
constexpr int kTileCols = 16;           // columns per workgroup
constexpr int kTileRows = 16;           // rows of V per step
constexpr int kTileMaxGroups = 4;       // groups of 64 x per wave
constexpr int kTileMaxD = 8 * kTileMaxGroups * 64;  // with 8 waves
static constexpr size_t tile_lds_bytes(int waves, int groups) {
  return sizeof(float) * (size_t)(waves * kTileRows * (64 * groups + 4) + 2 * waves * 256);
}

// kTileGroups: groups per wave, the same for all four waves (a group that lies beyond d is all zeros: its
// fetches are out of the buffers' range, so it costs matrix instructions but no branch).
// NW: waves per workgroup, 4 for d <= 1024, 8 (two per SIMD) for d <= 2048.
template <int NW, int kTileGroups>
__global__ void __launch_bounds__(64 * NW) chain_tile_kernel(ChainArgs p) {
  constexpr int kTileLd = 64 * kTileGroups + 4;  // row stride of a wave's slice in LDS (floats)
  extern __shared__ float smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = lane >> 4, i = lane & 15;
  const int d = p.d, m = p.m, n = p.n, k = p.k, kp = p.kp;
  const int col = blockIdx.x * kTileCols + i;
  const bool col_ok = col < m;
  float* Vw = smem + (size_t)wave * kTileRows * kTileLd;         // this wave's slice of the step's rows: [16][kTileLd]
  float* Bp = smem + (size_t)NW * kTileRows * kTileLd;           // partial products: [2][NW][256]
  auto group_x = [&](int g) { return 64 * (wave + NW * g); };

  // Input tile through a buffer bounded by the rows that exist: rows beyond them, columns beyond m and groups
  // this wave does not own read as zero without a branch, so all fetches are in flight together.
  f32x4 A[4 * kTileGroups];
  const BufferDesc xdesc = make_buffer(p.in, (size_t)p.in_rows * m * sizeof(float));
#pragma unroll
  for (int g = 0; g < kTileGroups; ++g) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int x = group_x(g) + 16 * q + 4 * j + r;
        const unsigned off = col_ok ? ((unsigned)x * (unsigned)m + (unsigned)col) * 4u : kOob;
        A[4 * g + r][j] = buffer_load<1>(xdesc, off, 0).e[0];
      }
    }
  }
  if (p.in_scale_mode) {
    const BufferDesc sdesc = make_buffer(p.in_scale, (size_t)p.in_rows * sizeof(float));
    f32x4 sg[4 * kTileGroups];
#pragma unroll
    for (int g = 0; g < kTileGroups; ++g) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int x = group_x(g) + 16 * q + 4 * j + r;
          sg[4 * g + r][j] = buffer_load<1>(sdesc, (unsigned)x * 4u, 0).e[0];
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    // The mode as a compile-time constant, and no branch per element: rows that do not exist hold zero in A
    // already; their sigma is replaced by 1 so that the factor stays finite.
    auto scale_rows = [&](auto mode) {
#pragma unroll
      for (int g = 0; g < kTileGroups; ++g) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int x = group_x(g) + 16 * q + 4 * j + r;
            const float sv = x < p.in_rows ? sg[4 * g + r][j] : 1.f;
            A[4 * g + r][j] *= diag_factor(decltype(mode)::value, sv);
          }
        }
      }
    };
    switch (p.in_scale_mode) {
      case 1: scale_rows(std::integral_constant<int, 1>()); break;
      case 2: scale_rows(std::integral_constant<int, 2>()); break;
      case 3: scale_rows(std::integral_constant<int, 3>()); break;
      default: scale_rows(std::integral_constant<int, 4>()); break;
    }
  }

  // staging of a step's 16 rows: lane l fetches 16 bytes at x = group_x(l / 16) + 4 (l % 16) of every row
  const BufferDesc vdesc = make_buffer(p.V, (size_t)n * d * sizeof(float));
  const int stage_x = group_x(lane >> 4) + 4 * (lane & 15);
  const unsigned stage_off = ((lane >> 4) < kTileGroups && stage_x < d) ? (unsigned)stage_x * 4u : kOob;
  BufVec<4> stage[kTileRows];
  auto fetch_rows = [&](int row0) {
#pragma unroll
    for (int rr = 0; rr < kTileRows; ++rr)
      stage[rr] = buffer_load<4>(vdesc, stage_off, (unsigned)(row0 + rr) * (unsigned)d * 4u);
  };
  auto stash_rows = [&]() {
    float* dst = Vw + 4 * lane;
#pragma unroll
    for (int rr = 0; rr < kTileRows; ++rr) {
      if (kTileGroups == 4 || (lane >> 4) < kTileGroups) lds_store<4>(dst + rr * kTileLd, stage[rr]);  // a row holds 64 kTileGroups floats
    }
  };
  // op(T) of the step that starts at row0, as the A operand of C = op(T) B: lane (q, i) holds op(T)(i, 4 kk + q)
  auto fetch_t = [&](int blk, int part, float (&t)[4]) {
    const float* Tb = p.T + (size_t)blk * kp * kp + (size_t)part * kTileRows * (kp + 1);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) t[kk] = p.transpose ? Tb[(4 * kk + q) * kp + i] : Tb[i * kp + 4 * kk + q];
  };

  const int ns = n / kTileRows;
  auto row_of = [&](int s) { return p.transpose ? kTileRows * s : n - kTileRows * (s + 1); };
  // The rows of step s + 1 are fetched into registers during step s and replace those of step s in LDS once its
  // second product has read them; the factor of step s + 1 is fetched at the start of step s.
  // (blk, part): block and 16-row part of the current step, (blkn, partn) of the next; counters, no division.
  const int sub = k / kTileRows;
  int blk = p.transpose ? 0 : p.nb - 1, part = p.transpose ? 0 : sub - 1;
  float tcur[4], tnxt[4];
  fetch_rows(row_of(0));
  fetch_t(blk, part, tcur);
  stash_rows();
  fetch_rows(row_of(ns > 1 ? 1 : 0));
  for (int s = 0; s < ns; ++s) {
    const int row0 = row_of(s), cur = s & 1;
    int blkn = blk, partn = part;
    if (s + 1 < ns) {
      if (p.transpose) {
        if (++partn == sub) { partn = 0; ++blkn; }
      } else {
        if (--partn < 0) { partn = sub - 1; --blkn; }
      }
    }
    fetch_t(blkn, partn, tnxt);
    if (p.save_in && part == (p.transpose ? 0 : sub - 1)) {
      const BufferDesc adesc = make_buffer(p.save_in + (size_t)blk * m * d, (size_t)m * d * sizeof(float));
#pragma unroll
      for (int g = 0; g < kTileGroups; ++g) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int x = group_x(g) + 16 * q + 4 * j;
          const unsigned off = (col_ok && x < d) ? ((unsigned)col * (unsigned)d + (unsigned)x) * 4u : kOob;
          BufVec<4> v;
          v.e[0] = A[4 * g][j]; v.e[1] = A[4 * g + 1][j]; v.e[2] = A[4 * g + 2][j]; v.e[3] = A[4 * g + 3][j];
          buffer_store<4>(adesc, off, 0, v);
        }
      }
    }
    const float* Vc = Vw;
    // B (partial over this wave's x) = V_rows A: four independent accumulation chains
    f32x4 acc[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
    // operand fetches run two ahead of the matrix instructions that use them
    auto v1_at = [&](int t) {  // t = 4 g + j
      return *reinterpret_cast<const float4*>(Vc + i * kTileLd + 64 * (t >> 2) + 16 * q + 4 * (t & 3));
    };
    {
      float4 va = v1_at(0), vb = v1_at(1);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
      for (int t = 0; t < 4 * kTileGroups; ++t) {
        const int g = t >> 2, j = t & 3;
        const float4 v4 = va;
        va = vb;
        if (t + 2 < 4 * kTileGroups) vb = v1_at(t + 2);
        acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.x, A[4 * g][j], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.y, A[4 * g + 1][j], acc[1], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.z, A[4 * g + 2][j], acc[2], 0, 0, 0);
        acc[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.w, A[4 * g + 3][j], acc[3], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read ...
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);  // ... then four matrix instructions
      }
    }
    const f32x4 bpart = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    // element (row 4 kk + qq, column i) of a wave's partial sits at ((qq * 16 + i) * 4 + kk): the writes of a
    // wave hit 64 different banks and the operand fetch below is one 16-byte read per wave summed over
    float* bw = Bp + (size_t)(cur * NW + wave) * 256;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) bw[(jj * 16 + i) * 4 + q] = bpart[jj];
    lds_barrier();
    const float* br = Bp + (size_t)cur * NW * 256 + (q * 16 + i) * 4;
    float4 b = *reinterpret_cast<const float4*>(br);
#pragma unroll
    for (int w = 1; w < NW; ++w) {
      const float4 t4 = *reinterpret_cast<const float4*>(br + w * 256);
      b.x += t4.x; b.y += t4.y; b.z += t4.z; b.w += t4.w;
    }
    f32x4 C = f32x4{0.f, 0.f, 0.f, 0.f};
    C = __builtin_amdgcn_mfma_f32_16x16x4f32(tcur[0], b.x, C, 0, 0, 0);
    C = __builtin_amdgcn_mfma_f32_16x16x4f32(tcur[1], b.y, C, 0, 0, 0);
    C = __builtin_amdgcn_mfma_f32_16x16x4f32(tcur[2], b.z, C, 0, 0, 0);
    C = __builtin_amdgcn_mfma_f32_16x16x4f32(tcur[3], b.w, C, 0, 0, 0);
    if (p.save_c && wave == 0 && col_ok)
      *reinterpret_cast<float4*>(p.save_c + (size_t)col * n + row0 + 4 * q) = make_float4(C[0], C[1], C[2], C[3]);
    // A -= V_rows^T C: contraction slice s2 pairs K index q with row 4 q + s2, which is where lane (q, i) holds C
    auto v2_at = [&](int t) {  // t = 4 g + s2
      return *reinterpret_cast<const float4*>(Vc + (4 * q + (t & 3)) * kTileLd + 64 * (t >> 2) + 4 * i);
    };
    {
      const float cn[4] = {-C[0], -C[1], -C[2], -C[3]};
      float4 va = v2_at(0), vb = v2_at(1);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
      for (int t = 0; t < 4 * kTileGroups; ++t) {
        const int g = t >> 2, s2 = t & 3;
        const float4 v4 = va;
        va = vb;
        if (t + 2 < 4 * kTileGroups) vb = v2_at(t + 2);
        A[4 * g] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.x, cn[s2], A[4 * g], 0, 0, 0);
        A[4 * g + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.y, cn[s2], A[4 * g + 1], 0, 0, 0);
        A[4 * g + 2] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.z, cn[s2], A[4 * g + 2], 0, 0, 0);
        A[4 * g + 3] = __builtin_amdgcn_mfma_f32_16x16x4f32(v4.w, cn[s2], A[4 * g + 3], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
    }
    stash_rows();
    fetch_rows(row_of(s + 2 < ns ? s + 2 : s));
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) tcur[kk] = tnxt[kk];
    blk = blkn; part = partn;
  }
  const BufferDesc odesc = make_buffer(p.out, (size_t)d * m * sizeof(float));
#pragma unroll
  for (int g = 0; g < kTileGroups; ++g) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int x = group_x(g) + 16 * q + 4 * j + r;
        const unsigned off = col_ok ? ((unsigned)x * (unsigned)m + (unsigned)col) * 4u : kOob;
        BufVec<1> v;
        v.e[0] = A[4 * g + r][j];
        buffer_store<1>(odesc, off, 0, v);
      }
    }
  }
}

// Shapes the matrix-core chain serves, and from how many columns on it is the faster one.
#ifndef FASTH_TILE_MIN_COLS
#define FASTH_TILE_MIN_COLS 769  // the per-column kernel needs a fourth round of 256 workgroups from here on
#endif
static bool chain_uses_tile(const ChainArgs& a) {
  return a.m >= FASTH_TILE_MIN_COLS && a.d % 4 == 0 && a.d <= kTileMaxD && a.k % kTileRows == 0 &&
         (size_t)a.d * a.m * sizeof(float) < kOob;  // its buffers take 32-bit byte offsets
}

static int launch_chain_tile(const ChainArgs& a, hipStream_t stream) {
  if (a.d > kTileMaxD || a.d % 4 != 0 || a.k % kTileRows != 0 || a.n % a.k != 0 ||
      (size_t)a.d * a.m * sizeof(float) >= kOob || (size_t)a.n * a.d * sizeof(float) >= kOob)
    return FASTH_EINVAL;
  const dim3 grid((a.m + kTileCols - 1) / kTileCols);
#define FASTH_LAUNCH_TILE(WW, GG)                                                                           \
  do {                                                                                                      \
    int rc_ = allow_lds(chain_tile_kernel<WW, GG>, tile_lds_bytes(WW, GG));                                 \
    if (rc_ != FASTH_OK) return rc_;                                                                        \
    prof::Scope ps_(FASTH_KERNEL_CHAIN, stream);                                                            \
    hipLaunchKernelGGL((chain_tile_kernel<WW, GG>), grid, dim3(64 * WW), tile_lds_bytes(WW, GG), stream, a); \
  } while (0)
  if (a.d <= 1024) {
    const int groups = (a.d + 255) / 256;  // per wave
    if (groups <= 1) FASTH_LAUNCH_TILE(4, 1);
    else if (groups == 2) FASTH_LAUNCH_TILE(4, 2);
    else if (groups == 3) FASTH_LAUNCH_TILE(4, 3);
    else FASTH_LAUNCH_TILE(4, 4);
  } else {
    const int groups = (a.d + 511) / 512;
    if (groups <= 3) FASTH_LAUNCH_TILE(8, 3);
    else FASTH_LAUNCH_TILE(8, 4);
  }
#undef FASTH_LAUNCH_TILE
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

// ---- Streaming chain kernel ----------------------------------------------------------------
// Any k <= 128 and any d <= VW * NT. The block is too large for registers, so its rows pass
// through them eight at a time, twice per block (once per product); the second read comes from
// the L2. The next group of rows is fetched while the current one is used.
template <int VW, int NT>
__global__ void __launch_bounds__(NT) chain_stream_kernel(ChainArgs p) {
  extern __shared__ float smem[];
  constexpr int NW = NT / 64, R = 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = blockIdx.x, m = p.m, d = p.d, k = p.k, kp = p.kp;
  const int LDT = kp + 4;
  float* Ts = smem;               // [kp][LDT]: op(T_i), row-contiguous
  float* Bpart = Ts + kp * LDT;   // [NW][kp]
  float* Bv = Bpart + NW * kp;    // [kp]
  float* Cpart = Bv + kp;         // [8][kp]
  float* Cv = Cpart + 8 * kp;     // [kp]
  const bool ok = VW * tid < d;
  const unsigned x0 = ok ? VW * tid : 0;
  Chunk<VW> a = load_column_chunk<VW>(p, col, x0, ok);
  const int sel = reduce_sel<R>(lane);
  const int ngroups = (k + R - 1) / R;
  // matvec work split: mg threads per row of T, each over kp / mg columns
  int mg = NT / kp < 8 ? NT / kp : 8;
  if (mg > kp / 4) mg = kp / 4;
  const int mrow = tid / mg, mpart = tid % mg, mlen = kp / mg;
  for (int s = 0; s < p.nb; ++s) {
    const int i = p.transpose ? s : p.nb - 1 - s;
    const float* Vi = p.V + (size_t)i * k * d + x0;
    const float* Ti = p.T + (size_t)i * kp * kp;
    for (int idx = tid; idx < kp * kp; idx += NT) {
      const int r = idx / kp, c = idx % kp;
      if (p.transpose) Ts[c * LDT + r] = Ti[idx];
      else Ts[r * LDT + c] = Ti[idx];
    }
    if (p.save_in && ok) store_chunk<VW>(p.save_in + ((size_t)i * m + col) * d + x0, a);
    auto load_group = [&](int g, Chunk<VW> (&rows)[R]) {
#pragma unroll
      for (int jj = 0; jj < R; ++jj) {
        const int j = min(g * R + jj, k - 1);  // rows past the block repeat its last row; their results are ignored
        rows[jj] = load_chunk<VW>(Vi + (size_t)j * d);
      }
    };
    auto dots = [&](int g, const Chunk<VW> (&rows)[R]) {
      float pj[R];
#pragma unroll
      for (int jj = 0; jj < R; ++jj) {
        float acc = 0.f;
#pragma unroll
        for (int r = 0; r < VW; ++r) acc = fmaf(rows[jj].e[r], a.e[r], acc);
        pj[jj] = acc;
      }
      wave_reduce_multi_reg<R>(pj);
      if ((lane & reduce_writer_mask<R>()) == 0) Bpart[wave * kp + g * R + sel] = pj[0];
    };
    Chunk<VW> ga[R], gb[R];
    load_group(0, ga);
    for (int g = 0; g < ngroups; g += 2) {
      if (g + 1 < ngroups) load_group(g + 1, gb);
      dots(g, ga);
      if (g + 1 < ngroups) {
        if (g + 2 < ngroups) load_group(g + 2, ga);
        dots(g + 1, gb);
      }
    }
    load_group(0, ga);  // first group of the second pass, in flight during the small products
    lds_barrier();
    if (tid < kp) {
      float b = 0.f;
      if (tid < k)
        for (int w = 0; w < NW; ++w) b += Bpart[w * kp + tid];
      Bv[tid] = b;
    }
    lds_barrier();
    if (mrow < kp) {
      const float* trow_ptr = Ts + mrow * LDT + mpart * mlen;
      const float* bptr = Bv + mpart * mlen;
      float c = 0.f;
      for (int l = 0; l < mlen; l += 4) {
        const float4 t4 = *reinterpret_cast<const float4*>(trow_ptr + l);
        const float4 b4 = *reinterpret_cast<const float4*>(bptr + l);
        c = fmaf(t4.x, b4.x, c); c = fmaf(t4.y, b4.y, c); c = fmaf(t4.z, b4.z, c); c = fmaf(t4.w, b4.w, c);
      }
      Cpart[mpart * kp + mrow] = c;
    }
    lds_barrier();
    if (tid < kp) {
      float c = 0.f;
      for (int g = 0; g < mg; ++g) c += Cpart[g * kp + tid];
      if (tid >= k) c = 0.f;
      Cv[tid] = c;
      if (p.save_c && tid < k) p.save_c[(size_t)col * p.n + (size_t)i * k + tid] = c;
    }
    lds_barrier();
    auto update = [&](int g, const Chunk<VW> (&rows)[R]) {
#pragma unroll
      for (int jj = 0; jj < R; ++jj) {
        const float c = Cv[g * R + jj];  // zero for rows past the block
#pragma unroll
        for (int r = 0; r < VW; ++r) a.e[r] = fmaf(-c, rows[jj].e[r], a.e[r]);
      }
    };
    for (int g = 0; g < ngroups; g += 2) {
      if (g + 1 < ngroups) load_group(g + 1, gb);
      update(g, ga);
      if (g + 1 < ngroups) {
        if (g + 2 < ngroups) load_group(g + 2, ga);
        update(g + 1, gb);
      }
    }
    if (!ok) {
#pragma unroll
      for (int r = 0; r < VW; ++r) a.e[r] = 0.f;
    }
    lds_barrier();  // Ts, Bpart and Cv are rewritten by the next block
  }
  if (ok) {
#pragma unroll
    for (int r = 0; r < VW; ++r) p.out[(size_t)(x0 + r) * m + col] = a.e[r];
  }
}

template <int VW, int NT>
static int launch_chain_stream(const ChainArgs& a, hipStream_t stream) {
  const size_t lds = sizeof(float) * ((size_t)a.kp * (a.kp + 4) + (size_t)(NT / 64) * a.kp + 10 * (size_t)a.kp);
  int rc = allow_lds(chain_stream_kernel<VW, NT>, lds);
  if (rc != FASTH_OK) return rc;
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream);
  hipLaunchKernelGGL((chain_stream_kernel<VW, NT>), dim3(a.m), dim3(NT), lds, stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

template <int VW>
static int launch_chain_stream_vw(const ChainArgs& a, hipStream_t stream) {
  const int chunks = a.d / VW;
  if (chunks <= 256) return launch_chain_stream<VW, 256>(a, stream);
  if (chunks <= 512) return launch_chain_stream<VW, 512>(a, stream);
  return launch_chain_stream<VW, 1024>(a, stream);
}

static bool chain_takes_side_product(const ChainArgs& a) {
  return !chain_uses_tile(a) && a.d % 4 == 0 && a.d <= 4096;
}

static int launch_chain_kernel(const ChainArgs& a, hipStream_t stream) {
  const int d = a.d, k = a.k;
  if (chain_uses_tile(a)) return launch_chain_tile(a, stream);
  if (chain_takes_side_product(a)) {  // every launch in this branch is a chain_pipe_kernel
    // whole block in registers, two copies; a quarter of the next block is fetched during the reduction
    if (k == 16 && d <= 1024) return launch_chain_pipe<16, 4, 256, 4>(a, stream);
    if (k == 16 && d <= 2048) return launch_chain_pipe<16, 4, 512, 4>(a, stream);
    if (k == 32 && d <= 256) return launch_chain_pipe<32, 1, 256, 8>(a, stream);
    if (k == 32 && d <= 512) return launch_chain_pipe<32, 2, 256, 8>(a, stream);
    // (10 of the 32 rows of the next block fetched during the first product, 8 during the reduction, 14 during
    // the update: with 12 / 8 / 12 more of the second register copy spills to the accumulator file; 117.2 -> 115.8 us
    // per forward + backward at d = n = 1024, m = 32)
    if (k == 32 && d <= 1024) return launch_chain_pipe<32, 4, 256, 8, 1, false, 10>(a, stream);
    if (k == 64 && d <= 256) return launch_chain_pipe<64, 1, 256, 16>(a, stream);
    if (k == 64 && d <= 512) return launch_chain_pipe<64, 2, 256, 16>(a, stream);
    // Larger blocks and longer vectors: two register copies of the whole block do not fit, but the block can be
    // applied as steps of 32 rows (d <= 1024) or 16 rows (d <= 2048, two waves per SIMD), which is faster than
    // one copy refilled in place or rows streamed twice (d = n = 2048: 178 us for k = 32, 64 and 128 alike,
    // against 222, 359 and 406 us)
    if (d <= 1024) {
      if (k == 64) return launch_chain_pipe<32, 4, 256, 8, 2, false, 10>(a, stream);
      if (k == 128) return launch_chain_pipe<32, 4, 256, 8, 4, false, 10>(a, stream);
      if (k == 8) return launch_chain_pipe<8, 4, 256, 2>(a, stream);
      // any other block size: steps of 8, 16 or 32 rows, the last one of a block short
      if (k < 8) return launch_chain_pipe<8, 4, 256, 2, 0, true>(a, stream);
      if (k < 16) return launch_chain_pipe<16, 4, 256, 4, 0, true>(a, stream);
      return launch_chain_pipe<32, 4, 256, 8, 0, true>(a, stream);
    } else if (d <= 2048) {
      if (k == 32) return launch_chain_pipe<16, 4, 512, 4, 2, false, 5>(a, stream);  // fetch split 5 / 4 / 7
      if (k == 64) return launch_chain_pipe<16, 4, 512, 4, 4, false, 5>(a, stream);
      if (k == 128) return launch_chain_pipe<16, 4, 512, 4, 8, false, 5>(a, stream);
      if (k == 8) return launch_chain_pipe<8, 4, 512, 2>(a, stream);
      if (k < 8) return launch_chain_pipe<8, 4, 512, 2, 0, true>(a, stream);
      return launch_chain_pipe<16, 4, 512, 4, 0, true>(a, stream);
    } else {
      // 16 waves share 512 registers per lane: two copies of 8 rows
      if (k % 8 == 0) return launch_chain_pipe<8, 4, 1024, 2, 0>(a, stream);
      return launch_chain_pipe<8, 4, 1024, 2, 0, true>(a, stream);
    }
  }
  if (d % 2 == 0 && d <= 2048) return launch_chain_stream_vw<2>(a, stream);
  if (d <= 1024) return launch_chain_stream_vw<1>(a, stream);
  int threads = 256;
  if (d > 256 * 8) threads = 512;
  if (d > 512 * 8) threads = 1024;
  const int per = (d + threads - 1) / threads;
  const int nw = threads / 64;
  const size_t lds = sizeof(float) * ((size_t)a.kp * (a.kp + 1) + (size_t)nw * a.kp + 2 * a.kp);
  dim3 grid(a.m), block(threads);
#define FASTH_LAUNCH_CHAIN(UU)                                                   \
  do {                                                                           \
    int rc_ = allow_lds(chain_kernel<UU>, lds);                                  \
    if (rc_ != FASTH_OK) return rc_;                                             \
    prof::Scope ps_(FASTH_KERNEL_CHAIN, stream);                                 \
    hipLaunchKernelGGL(chain_kernel<UU>, grid, block, lds, stream, a);           \
  } while (0)
  if (per <= 1) FASTH_LAUNCH_CHAIN(1);
  else if (per <= 2) FASTH_LAUNCH_CHAIN(2);
  else if (per <= 4) FASTH_LAUNCH_CHAIN(4);
  else if (per <= 8) FASTH_LAUNCH_CHAIN(8);
  else FASTH_LAUNCH_CHAIN(16);
#undef FASTH_LAUNCH_CHAIN
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

static int launch_chain(const ChainArgs& a, hipStream_t stream) {
  const int rc = launch_chain_kernel(a, stream);
  if (rc != FASTH_OK || !a.ds_out || chain_takes_side_product(a)) return rc;
  prof::Scope ps_(FASTH_KERNEL_DSIGMA, stream);
  hipLaunchKernelGGL(dsigma_kernel, dim3((a.ds_rows + 3) / 4), dim3(256), 0, stream, a.in, a.ds_z1, a.in_scale, a.ds_out,
                     a.ds_rows, a.m, a.in_scale_mode);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

// ------------------------------------------------------------------------------------------
// Algorithm 2 Step 2, per block, as dense products (equal to summing Eq. 5 over the block's
// reflections and the mini-batch). With a = input of block i (saved by the activation chain),
// g = dL/d(output of block i) (saved by the gradient chain), Ca and Cg the two chains'
// coefficient matrices (k x m):
//   Z = Cg Ca^T (k x k);  E = sym(striu(Z)) + diag(Z)   for A = H X
//                         E = sym(stril(Z)) + diag(Z)   for A = H^T X
//   dV_i = -(Ca g^T + Cg a^T) + E V_i
// grid (ceil(d / 64), nb), 256 threads. With few columns every workgroup rebuilds the small matrix Z on its
// way over the mini-batch (2 k^2 m FLOP each, no extra launch); with many (k >= 64 and k m >= 32768)
// dv_z_kernel forms the Z of every block once and the workgroups read it (PREZ).
// ------------------------------------------------------------------------------------------

struct DvArgs {
  const float* V;       // [n][d]
  const float* saveA;   // [nb][m][d]
  const float* saveCa;  // [m][n]
  const float* saveG;   // [nb][m][d]
  const float* saveCg;  // [m][n]
  float* dV;            // [n][d]
  float* Z;             // [nb][kp][kp]: Z = Cg Ca^T per block when it is formed by dv_z_kernel
  int d, n, m, k, kp;
  int transpose;        // of the forward product
  int accumulate;       // add to dV instead of overwriting it (a factor that enters a layer twice)
};

// Up to two products per launch (the two factors of an SVD layer): blockIdx.z picks the product.
struct DvPair {
  DvArgs a[2];
};

// Z_i = Cg_i Ca_i^T for every block: one workgroup per 16 x 16 tile of Z_i, grid (kt^2, nb, products). The four
// waves split the mini-batch columns (wave w takes columns 16 c + 4 w .. + 3) and their partial tiles meet in
// LDS. Operands come straight from the coefficient matrices [m][n]: lane (q, li) needs Cg(16 ti + li, col + q)
// and Ca(16 tj + li, col + q), 16 consecutive floats per q.
__global__ void __launch_bounds__(256) dv_z_kernel(DvPair pair) {
  __shared__ __align__(16) float part[4][256];
  const DvArgs p = pair.a[blockIdx.z];
  const int k = p.k, kp = p.kp, m = p.m, n = p.n, kt = kp / 16;
  if ((int)blockIdx.y * k >= n || (int)blockIdx.x >= kt * kt) return;  // whole workgroup, before the barrier
  const int i = blockIdx.y, ti = blockIdx.x / kt, tj = blockIdx.x % kt;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, q = lane >> 4;
  const BufferDesc cgdesc = make_buffer(p.saveCg, (size_t)m * n * sizeof(float));
  const BufferDesc cadesc = make_buffer(p.saveCa, (size_t)m * n * sizeof(float));
  const bool g_ok = 16 * ti + li < k, a_ok = 16 * tj + li < k;  // rows of the padding read as zero
  const unsigned g_row = (unsigned)(i * k + 16 * ti + li) * 4u, a_row = (unsigned)(i * k + 16 * tj + li) * 4u;
  constexpr int UN = 8;  // column groups in flight per wave
  f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
  for (int c0 = 4 * wave; c0 < m; c0 += 16 * UN) {
    float a[UN], b[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int col = c0 + 16 * u + q;
      const unsigned off = (unsigned)col * (unsigned)n * 4u;
      a[u] = buffer_load<1>(cgdesc, (col < m && g_ok) ? off + g_row : kOob, 0).e[0];
      b[u] = buffer_load<1>(cadesc, (col < m && a_ok) ? off + a_row : kOob, 0).e[0];
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) acc[u & 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u], b[u], acc[u & 1], 0, 0, 0);
  }
  const f32x4 z = acc[0] + acc[1];
  *reinterpret_cast<float4*>(&part[wave][4 * lane]) = make_float4(z[0], z[1], z[2], z[3]);
  __syncthreads();
  if (wave == 0) {
    float* Zi = p.Z + (size_t)i * kp * kp;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const float v = (part[0][4 * lane + jj] + part[1][4 * lane + jj]) + (part[2][4 * lane + jj] + part[3][4 * lane + jj]);
      Zi[(16 * ti + 4 * q + jj) * kp + 16 * tj + li] = v;
    }
  }
}

template <int KT, int VEC, bool PREZ>  // kp = 16 KT; VEC = 4 when d is a multiple of 4 (16-byte loads along x), else 1
__global__ void __launch_bounds__(256) dv_kernel(DvPair pair) {
  extern __shared__ __align__(16) float smem[];
  constexpr int kp = 16 * KT;
  const DvArgs p = pair.a[blockIdx.z];
  const int k = p.k, d = p.d, m = p.m, n = p.n;
  if ((int)blockIdx.y * k >= n || (int)blockIdx.x * kDvTile >= d) return;  // whole workgroup, before any barrier
  constexpr int LDE = kp + 4, LDC = kDvMChunk + 4, LDX = kDvTile + 4;
  float* Es = smem;                   // [kp][LDE]
  float* Cas = Es + kp * LDE;         // [kp][LDC]
  float* Cgs = Cas + kp * LDC;        // [kp][LDC]
  float* gT = Cgs + kp * LDC;         // [kDvMChunk][LDX]
  float* aT = gT + kDvMChunk * LDX;   // [kDvMChunk][LDX]
  float* Vs = aT + kDvMChunk * LDX;   // [kp][LDX]
  const int i = blockIdx.y, x0 = blockIdx.x * kDvTile;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, q = lane >> 4;
  constexpr int kt = KT;
  constexpr int XV = kDvTile / VEC;                    // loads per tile row
  constexpr int V_PER = kp * kDvTile / VEC / 256;      // loads of the V tile per thread
  constexpr int X_PER = kDvMChunk * kDvTile / VEC / 256;  // loads of the a^T / g^T tile per thread
  constexpr int C_PER = kp * kDvMChunk / 256;          // loads of each coefficient tile per thread

  // All fetches go through buffers whose size is the valid extent, so nothing branches on a bound
  // and the fetches of a tile are in flight together. The block's rows of V are needed last; they
  // are fetched first so that one trip to memory covers them and the first mini-batch chunk.
  BufVec<VEC> vreg[V_PER];
  {
    const BufferDesc vdesc = make_buffer(p.V + (size_t)i * k * d, (size_t)k * d * sizeof(float));
#pragma unroll
    for (int it = 0; it < V_PER; ++it) {
      const int idx = tid + it * 256, j = idx / XV, x = x0 + (idx % XV) * VEC;
      vreg[it] = buffer_load<VEC>(vdesc, x < d ? (unsigned)(j * d + x) * 4u : kOob, 0);  // rows >= k lie beyond the buffer
    }
  }
  struct Chunk {
    BufVec<VEC> g[X_PER], a[X_PER];
    float ca[C_PER], cg[C_PER];
  };
  auto fetch = [&](int mc, Chunk& c) {
    const int rows = min(kDvMChunk, m - mc);  // mini-batch columns in this chunk
    const BufferDesc gdesc = make_buffer(p.saveG + ((size_t)i * m + mc) * d, (size_t)rows * d * sizeof(float));
    const BufferDesc adesc = make_buffer(p.saveA + ((size_t)i * m + mc) * d, (size_t)rows * d * sizeof(float));
    const BufferDesc cadesc = make_buffer(p.saveCa + (size_t)mc * n, (size_t)rows * n * sizeof(float));
    const BufferDesc cgdesc = make_buffer(p.saveCg + (size_t)mc * n, (size_t)rows * n * sizeof(float));
#pragma unroll
    for (int it = 0; it < X_PER; ++it) {
      const int idx = tid + it * 256, lc = idx / XV, x = x0 + (idx % XV) * VEC;
      const unsigned off = x < d ? (unsigned)(lc * d + x) * 4u : kOob;
      c.g[it] = buffer_load<VEC>(gdesc, off, 0);
      c.a[it] = buffer_load<VEC>(adesc, off, 0);
    }
#pragma unroll
    for (int it = 0; it < C_PER; ++it) {
      const int idx = tid + it * 256, j = idx % kp, lc = idx / kp;
      const unsigned off = j < k ? (unsigned)(lc * n + i * k + j) * 4u : kOob;
      c.ca[it] = buffer_load<1>(cadesc, off, 0).e[0];
      c.cg[it] = buffer_load<1>(cgdesc, off, 0).e[0];
    }
  };
  auto to_lds = [&](const Chunk& c) {
#pragma unroll
    for (int it = 0; it < X_PER; ++it) {
      const int idx = tid + it * 256, lc = idx / XV, xv = (idx % XV) * VEC;
      lds_store<VEC>(gT + lc * LDX + xv, c.g[it]);
      lds_store<VEC>(aT + lc * LDX + xv, c.a[it]);
    }
#pragma unroll
    for (int it = 0; it < C_PER; ++it) {
      const int idx = tid + it * 256, j = idx % kp, lc = idx / kp;
      Cas[j * LDC + lc] = c.ca[it];
      Cgs[j * LDC + lc] = c.cg[it];
    }
  };
  Chunk cur;
  fetch(0, cur);
#pragma unroll
  for (int it = 0; it < V_PER; ++it) {
    const int idx = tid + it * 256;
    lds_store<VEC>(Vs + (idx / XV) * LDX + (idx % XV) * VEC, vreg[it]);
  }

  // One pass over the mini-batch accumulates both Z = Cg Ca^T and Ca g^T + Cg a^T.
  constexpr int kMaxZ = (KT * KT + 3) / 4;  // Z tiles per wave
  constexpr int kMaxAcc = KT;               // KT x 4 output tiles over 4 waves
  // The contraction over a chunk's 32 columns may run in any order: lane (q, li) takes columns 8 q .. 8 q + 7, so
  // an operand that is contiguous along the columns (the coefficient tiles) comes as two 16-byte LDS reads per
  // 8 matrix instructions. A wave's output tiles all lie in x tile `wave` (t = wave + 4 w), so its g^T / a^T
  // operands are fetched once per chunk and serve all KT row tiles. The two terms of a tile accumulate
  // separately (two independent chains of matrix instructions) and are added at the end.
  static_assert(kDvMChunk == 32, "column order of the contraction");
  auto row8 = [&](const float* base, float (&v)[8]) {
    const float4 lo = *reinterpret_cast<const float4*>(base), hi = *reinterpret_cast<const float4*>(base + 4);
    v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
  };
  f32x4 z[kMaxZ], acc[kMaxAcc], acc2[kMaxAcc];
#pragma unroll
  for (int w = 0; w < kMaxZ; ++w) z[w] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int w = 0; w < kMaxAcc; ++w) acc[w] = acc2[w] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int mc = 0; mc < m; mc += kDvMChunk) {
    if (mc) __syncthreads();
    to_lds(cur);
    __syncthreads();
    if (mc + kDvMChunk < m) fetch(mc + kDvMChunk, cur);  // in flight during this chunk's products
    if constexpr (!PREZ) {
#pragma unroll
      for (int w = 0; w < kMaxZ; ++w) {
        const int t = wave + 4 * w;
        if (t < kt * kt) {
          const int ti = t / kt, tj = t % kt;
          float cg[8], ca[8];
          row8(Cgs + (ti * 16 + li) * LDC + 8 * q, cg);
          row8(Cas + (tj * 16 + li) * LDC + 8 * q, ca);
#pragma unroll
          for (int kk = 0; kk < 8; ++kk) z[w] = __builtin_amdgcn_mfma_f32_16x16x4f32(cg[kk], ca[kk], z[w], 0, 0, 0);
        }
      }
    }
    float bg[8], ba[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      bg[kk] = gT[(8 * q + kk) * LDX + wave * 16 + li];
      ba[kk] = aT[(8 * q + kk) * LDX + wave * 16 + li];
    }
#pragma unroll
    for (int w = 0; w < kMaxAcc; ++w) {  // row tile ti = w, x tile = wave
      float ca[8], cg[8];
      row8(Cas + (w * 16 + li) * LDC + 8 * q, ca);
      row8(Cgs + (w * 16 + li) * LDC + 8 * q, cg);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        acc[w] = __builtin_amdgcn_mfma_f32_16x16x4f32(ca[kk], bg[kk], acc[w], 0, 0, 0);
        acc2[w] = __builtin_amdgcn_mfma_f32_16x16x4f32(cg[kk], ba[kk], acc2[w], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int w = 0; w < kMaxAcc; ++w) acc[w] += acc2[w];
  // E: mirror the triangle of Z that carries the gradient of T_i^-1. The matrix-core layout gives
  // lane (q, li) the entries Z(16 ti + 4 q + jj, 16 tj + li); each is written to its own place and,
  // if it lies in the carrying triangle, to the mirrored place as well.
  if constexpr (PREZ) {
    const float* Zi = p.Z + (size_t)i * kp * kp;
    for (int idx = tid; idx < kp * kp; idx += 256) {
      const int r = idx / kp, c = idx % kp;
      const bool own = p.transpose ? (r >= c) : (r <= c);  // the entry itself carries, else its mirror image does
      Es[r * LDE + c] = own ? Zi[r * kp + c] : Zi[c * kp + r];
    }
  } else {
#pragma unroll
    for (int w = 0; w < kMaxZ; ++w) {
      const int t = wave + 4 * w;
      if (t < kt * kt) {
        const int ti = t / kt, tj = t % kt;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int r = ti * 16 + 4 * q + jj, c = tj * 16 + li;
          const bool carries = p.transpose ? (r > c) : (r < c);
          if (carries) {
            Es[r * LDE + c] = z[w][jj];
            Es[c * LDE + r] = z[w][jj];
          } else if (r == c) {
            Es[r * LDE + c] = z[w][jj];
          }
        }
      }
    }
  }
  __syncthreads();
  // dV_i = -(Ca g^T + Cg a^T) + E V_i
#pragma unroll
  for (int w = 0; w < kMaxAcc; ++w) {
    const int t = wave + 4 * w;
    if (t < kt * 4) {
      const int ti = t / 4, tx = t % 4;
      f32x4 ev = {0.f, 0.f, 0.f, 0.f};
      ev = tile_mma(Es + ti * 16 * LDE, LDE, 1, Vs + tx * 16, LDX, 1, kp, ev);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int j = ti * 16 + 4 * q + jj, x = x0 + tx * 16 + li;
        if (j < k && x < d) {
          float* dst = p.dV + ((size_t)i * k + j) * d + x;
          const float val = ev[jj] - acc[w][jj];
          *dst = p.accumulate ? *dst + val : val;
        }
      }
    }
  }
}

static size_t dv_lds(int kp) {
  return sizeof(float) * ((size_t)kp * (kp + 4) + 2 * (size_t)kp * (kDvMChunk + 4) +
                          2 * (size_t)kDvMChunk * (kDvTile + 4) + (size_t)kp * (kDvTile + 4));
}

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
  for (int s = 0; s < n; ++s) {
    const int j = transpose ? s : n - 1 - s;
    const float* vr = V + (size_t)j * d;
    float v[U];
    float r[2] = {0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int x = tid + u * nthreads;
      v[u] = x < d ? vr[x] : 0.f;
      r[0] += v[u] * a[u];
      r[1] += v[u] * v[u];
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
  for (int s = 0; s < n; ++s) {
    const int j = transpose ? n - 1 - s : s;
    const float* vr = V + (size_t)j * d;
    float v[U];
    float r[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int x = tid + u * nthreads;
      v[u] = x < d ? vr[x] : 0.f;
      r[0] += v[u] * a[u];
      r[1] += v[u] * g[u];
      r[2] += v[u] * v[u];
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

// ------------------------------------------------------------------------------------------
// Host drivers
// ------------------------------------------------------------------------------------------

struct Product {  // one Householder product bound to its slice of a workspace
  int d, n, m, k;
  Layout L;
  char* ws;
  float* T() const { return reinterpret_cast<float*>(ws + L.off_T); }
  float* Spart() const { return reinterpret_cast<float*>(ws + L.off_Spart); }
  float* saveA() const { return reinterpret_cast<float*>(ws + L.off_saveA); }
  float* saveCa() const { return reinterpret_cast<float*>(ws + L.off_saveCa); }
  float* saveG() const { return reinterpret_cast<float*>(ws + L.off_saveG); }
  float* saveCg() const { return reinterpret_cast<float*>(ws + L.off_saveCg); }
};

static Product bind(int d, int n, int m, int k, void* ws) {
  Product P;
  P.d = d; P.n = n; P.m = m; P.k = k;
  P.L = make_layout(d, n, m, k);
  P.ws = static_cast<char*>(ws);
  return P;
}

static int launch_factor_fused(const FactorPair& fp, int count, int kp, bool vec4, hipStream_t stream) {
  prof::Scope ps_(FASTH_KERNEL_FACTOR, stream);
  const dim3 grid(count == 2 && fp.nb[1] > fp.nb[0] ? fp.nb[1] : fp.nb[0], count), block(512);
  if (vec4) {
    if (kp == 16) hipLaunchKernelGGL((factor_fused_kernel<1, 4>), grid, block, 0, stream, fp);
    else hipLaunchKernelGGL((factor_fused_kernel<2, 4>), grid, block, 0, stream, fp);
  } else {
    if (kp == 16) hipLaunchKernelGGL((factor_fused_kernel<1, 1>), grid, block, 0, stream, fp);
    else hipLaunchKernelGGL((factor_fused_kernel<2, 1>), grid, block, 0, stream, fp);
  }
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

static void set_factor_slot(FactorPair& fp, int slot, const Product& P, const float* V) {
  fp.V[slot] = V; fp.T[slot] = P.T(); fp.d[slot] = P.d; fp.k[slot] = P.k; fp.nb[slot] = P.L.nb;
}

static int build_factors(const Product& P, const float* V, hipStream_t stream) {
  const int kp = P.L.kp;
  if (kp <= 32) {
    FactorPair fp;
    set_factor_slot(fp, 0, P, V);
    set_factor_slot(fp, 1, P, V);  // unused
    return launch_factor_fused(fp, 1, kp, P.d % 4 == 0, stream);
  }
  {
    const size_t lds = sizeof(float) * (size_t)kp * (kGramChunk + 4);
    int rc = allow_lds(gram_partial_kernel<4>, lds);
    if (rc == FASTH_OK) rc = allow_lds(gram_partial_kernel<1>, lds);
    if (rc != FASTH_OK) return rc;
    prof::Scope ps_(FASTH_KERNEL_GRAM, stream);
    const dim3 grid(P.L.gram_split, P.L.nb);
    if (P.d % 4 == 0)
      hipLaunchKernelGGL(gram_partial_kernel<4>, grid, dim3(256), lds, stream, V, P.Spart(), P.d, P.k, kp, P.L.gram_split);
    else
      hipLaunchKernelGGL(gram_partial_kernel<1>, grid, dim3(256), lds, stream, V, P.Spart(), P.d, P.k, kp, P.L.gram_split);
    FASTH_HIP(hipGetLastError());
  }
  {
    const size_t lds = t_build_lds(kp);
    int rc = allow_lds(t_build_kernel, lds);
    if (rc != FASTH_OK) return rc;
    prof::Scope ps_(FASTH_KERNEL_TBUILD, stream);
    hipLaunchKernelGGL(t_build_kernel, dim3(P.L.nb), dim3(kp >= 128 ? 1024 : kp >= 64 ? 512 : 256), lds, stream, P.Spart(), P.T(), P.k, kp, P.L.gram_split);
    FASTH_HIP(hipGetLastError());
  }
  return FASTH_OK;
}

// Factors of two products (independent of each other) in one launch when both take the fused
// kernel with the same template arguments; otherwise one after the other.
static int build_factors_pair(const Product& P0, const float* V0, const Product& P1, const float* V1,
                              hipStream_t stream) {
  if (P0.L.kp <= 32 && P0.L.kp == P1.L.kp && (P0.d % 4 == 0) == (P1.d % 4 == 0)) {
    FactorPair fp;
    set_factor_slot(fp, 0, P0, V0);
    set_factor_slot(fp, 1, P1, V1);
    return launch_factor_fused(fp, 2, P0.L.kp, P0.d % 4 == 0, stream);
  }
  const int rc = build_factors(P0, V0, stream);
  return rc != FASTH_OK ? rc : build_factors(P1, V1, stream);
}

// A = H in (transpose = 0) or H^T in (transpose = 1); activation = true saves into the activation
// slots of the workspace, false into the gradient slots.
static int run_chain(const Product& P, const float* V, const float* in, float* out, int transpose, bool activation,
                     const float* in_scale, int in_scale_mode, hipStream_t stream, bool save = true,
                     const float* factors = nullptr, int in_rows = -1, const float* ds_z1 = nullptr,
                     float* ds_out = nullptr, int ds_rows = 0) {
  ChainArgs a;
  a.V = V; a.T = factors ? factors : P.T(); a.in = in; a.out = out;
  a.save_in = !save ? nullptr : activation ? P.saveA() : P.saveG();
  a.save_c = !save ? nullptr : activation ? P.saveCa() : P.saveCg();
  a.in_scale = in_scale; a.in_scale_mode = in_scale_mode;
  a.in_rows = in_rows < 0 ? P.d : in_rows;
  a.d = P.d; a.n = P.n; a.m = P.m; a.k = P.k; a.kp = P.L.kp; a.nb = P.L.nb;
  a.transpose = transpose;
  a.sub = 1;
  a.ds_z1 = ds_z1; a.ds_out = ds_out; a.ds_rows = ds_rows;
  return launch_chain(a, stream);
}

static DvArgs dv_args(const Product& P, const float* V, float* dV, int transpose, bool accumulate) {
  DvArgs a;
  a.accumulate = accumulate ? 1 : 0;
  a.V = V; a.saveA = P.saveA(); a.saveCa = P.saveCa(); a.saveG = P.saveG(); a.saveCg = P.saveCg(); a.dV = dV;
  a.Z = P.Spart();  // the partial Gram matrices are dead once the factors exist; Z needs nb kp^2 of their floats
  a.d = P.d; a.n = P.n; a.m = P.m; a.k = P.k; a.kp = P.L.kp; a.transpose = transpose;
  return a;
}

static int launch_dv(const DvPair& pair, int count, int kp, bool vec4, hipStream_t stream) {
  const size_t lds = dv_lds(kp);
  int xt = (pair.a[0].d + kDvTile - 1) / kDvTile, nb = pair.a[0].n / pair.a[0].k;
  if (count == 2) {
    xt = std::max(xt, (pair.a[1].d + kDvTile - 1) / kDvTile);
    nb = std::max(nb, pair.a[1].n / pair.a[1].k);
  }
  const dim3 grid(xt, nb, count);
  // Many columns and blocks of 64 rows or more: Z of every block once, by a launch of its own (measured at
  // d = n = 1024, m = 4096: dV 374 -> 326 us at k = 64, 853 -> 545 us at k = 128, but 294 -> 309 us at k = 32, where
  // the rebuild is a fifth of the work). Same condition for both products of a pair: they share m and k.
  const DvArgs& a0 = pair.a[0];
  const bool prez = a0.k >= 64 && (size_t)a0.m * a0.k >= 32768 && (size_t)a0.m * a0.n * sizeof(float) < kOob && a0.Z != nullptr &&
                    (count == 1 || (pair.a[1].m == a0.m && pair.a[1].k == a0.k && pair.a[1].Z != nullptr));
  prof::Scope ps_(FASTH_KERNEL_DV, stream);
  if (prez) {
    const int kt = kp / 16;
    hipLaunchKernelGGL(dv_z_kernel, dim3(kt * kt, nb, count), dim3(256), 0, stream, pair);
    FASTH_HIP(hipGetLastError());
  }
#define FASTH_LAUNCH_DV_(KT, VV, PZ)                                                      \
  do {                                                                                    \
    int rc_ = allow_lds(dv_kernel<KT, VV, PZ>, lds);                                      \
    if (rc_ != FASTH_OK) return rc_;                                                      \
    hipLaunchKernelGGL((dv_kernel<KT, VV, PZ>), grid, dim3(256), lds, stream, pair);      \
  } while (0)
#define FASTH_LAUNCH_DV(KT)                                                               \
  do {                                                                                    \
    if (vec4 && prez) FASTH_LAUNCH_DV_(KT, 4, true);                                      \
    else if (vec4) FASTH_LAUNCH_DV_(KT, 4, false);                                        \
    else if (prez) FASTH_LAUNCH_DV_(KT, 1, true);                                         \
    else FASTH_LAUNCH_DV_(KT, 1, false);                                                  \
  } while (0)
  switch (kp) {
    case 16: FASTH_LAUNCH_DV(1); break;
    case 32: FASTH_LAUNCH_DV(2); break;
    case 64: FASTH_LAUNCH_DV(4); break;
    default: FASTH_LAUNCH_DV(8); break;
  }
#undef FASTH_LAUNCH_DV
#undef FASTH_LAUNCH_DV_
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

static int run_dv(const Product& P, const float* V, float* dV, int transpose, hipStream_t stream,
                  bool accumulate = false) {
  DvPair pair;
  pair.a[0] = pair.a[1] = dv_args(P, V, dV, transpose, accumulate);
  return launch_dv(pair, 1, P.L.kp, P.d % 4 == 0, stream);
}

// dV of two products with different outputs in one launch when both take the same template
// arguments; otherwise one after the other.
static int run_dv_pair(const Product& P0, const float* V0, float* dV0, int transpose0, const Product& P1,
                       const float* V1, float* dV1, int transpose1, hipStream_t stream) {
  if (P0.L.kp == P1.L.kp && (P0.d % 4 == 0) == (P1.d % 4 == 0)) {
    DvPair pair;
    pair.a[0] = dv_args(P0, V0, dV0, transpose0, false);
    pair.a[1] = dv_args(P1, V1, dV1, transpose1, false);
    return launch_dv(pair, 2, P0.L.kp, P0.d % 4 == 0, stream);
  }
  const int rc = run_dv(P0, V0, dV0, transpose0, stream);
  return rc != FASTH_OK ? rc : run_dv(P1, V1, dV1, transpose1, stream);
}

static int seq_threads(int d) {
  int threads = 256;
  if (d > 256 * 8) threads = 512;
  if (d > 512 * 8) threads = 1024;
  return threads;
}

struct SvdLayout {
  size_t off_U, off_V, off_Z1, off_dZ2, total;
};

static SvdLayout make_svd_layout(int d, int n, int m, int k) {
  SvdLayout S;
  const size_t one = make_layout(d, n, m, k).total;
  S.off_U = 0;
  S.off_V = align_up(one, 256);
  S.off_Z1 = S.off_V + align_up(one, 256);
  S.off_dZ2 = S.off_Z1 + align_up((size_t)d * m * sizeof(float), 256);
  S.total = S.off_dZ2 + align_up((size_t)d * m * sizeof(float), 256);
  return S;
}

static int check_svd_shape(const fasth_svd_shape* s, fasth_shape* out) {
  if (!s) return FASTH_EINVAL;
  out->d = s->d; out->n = s->n; out->m = s->m; out->k = s->k; out->transpose = 0;
  return check_shape(out);
}

// Forward of the layer: first factor transposed, diagonal scale fused into the second chain's load.
static int svd_forward(const fasth_svd_shape* shape, const float* first, const float* sigma, const float* second,
                       const float* X, float* Y, void* workspace, size_t workspace_bytes, void* stream, int scale_mode) {
  fasth_shape fs;
  int rc = check_svd_shape(shape, &fs);
  if (rc != FASTH_OK) return rc;
  if (!first || !sigma || !second || !X || !Y || !workspace) return FASTH_EINVAL;
  if (!aligned16(first) || !aligned16(sigma) || !aligned16(second) || !aligned16(X) || !aligned16(Y) ||
      !aligned16(workspace))
    return FASTH_EALIGN;
  const SvdLayout S = make_svd_layout(fs.d, fs.n, fs.m, fs.k);
  if (workspace_bytes < S.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  // "first" is the factor applied transposed (V for W, U for W^-1); it owns slot off_V.
  const Product Pf = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_V);
  const Product Ps = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_U);
  float* Z1 = reinterpret_cast<float*>(ws + S.off_Z1);
  if ((rc = build_factors_pair(Pf, first, Ps, second, st)) != FASTH_OK) return rc;
  if ((rc = run_chain(Pf, first, X, Z1, 1, true, nullptr, 0, st)) != FASTH_OK) return rc;
  return run_chain(Ps, second, Z1, Y, 0, true, sigma, scale_mode, st);
}

static int svd_backward(const fasth_svd_shape* shape, const float* first, const float* sigma, const float* second,
                        const float* G, float* dfirst, float* dsigma, float* dsecond, float* dX, void* workspace,
                        size_t workspace_bytes, void* stream, int scale_mode) {
  fasth_shape fs;
  int rc = check_svd_shape(shape, &fs);
  if (rc != FASTH_OK) return rc;
  if (!first || !sigma || !second || !G || !dfirst || !dsigma || !dsecond || !dX || !workspace) return FASTH_EINVAL;
  if (!aligned16(first) || !aligned16(sigma) || !aligned16(second) || !aligned16(G) || !aligned16(dfirst) ||
      !aligned16(dsigma) || !aligned16(dsecond) || !aligned16(dX) || !aligned16(workspace))
    return FASTH_EALIGN;
  const SvdLayout S = make_svd_layout(fs.d, fs.n, fs.m, fs.k);
  if (workspace_bytes < S.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const Product Pf = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_V);
  const Product Ps = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_U);
  const float* Z1 = reinterpret_cast<const float*>(ws + S.off_Z1);
  float* dZ2 = reinterpret_cast<float*>(ws + S.off_dZ2);
  // through the second (plain) factor
  if ((rc = run_chain(Ps, second, G, dZ2, 1, false, nullptr, 0, st)) != FASTH_OK) return rc;
  // through the first (transposed) factor; dZ1 = s * dZ2 is fused into the chain's load, and the gradient of
  // sigma, which needs the same dZ2, rides along in the same launch
  if ((rc = run_chain(Pf, first, dZ2, dX, 0, false, sigma, scale_mode, st, true, nullptr, -1, Z1, dsigma, fs.d)) !=
      FASTH_OK)
    return rc;
  // both factors' vector gradients in one launch: each reads only its own saved slots
  return run_dv_pair(Ps, second, dsecond, 0, Pf, first, dfirst, 1, st);
}

static int sym_scale_mode(int function) {
  switch (function) {
    case FASTH_DIAG_IDENTITY: return 1;
    case FASTH_DIAG_EXP: return 3;
    case FASTH_DIAG_CAYLEY: return 4;
    default: return -1;
  }
}

// Rectangular layer (Section 3.3 "Rectangular Matrices"): U is rows x rows, V is cols x cols and
// Sigma is rows x cols with min(rows, cols) diagonal entries.
struct RectLayout {
  size_t off_U, off_V, off_Z1, off_dZ2, total;
};

static int check_rect_shape(const fasth_rect_shape* s, fasth_shape* u, fasth_shape* v) {
  if (!s) return FASTH_EINVAL;
  u->d = s->rows; u->n = s->n_u; u->m = s->m; u->k = s->k; u->transpose = 0;
  v->d = s->cols; v->n = s->n_v; v->m = s->m; v->k = s->k; v->transpose = 0;
  const int rc = check_shape(u);
  return rc != FASTH_OK ? rc : check_shape(v);
}

static RectLayout make_rect_layout(const fasth_shape& u, const fasth_shape& v) {
  RectLayout S;
  S.off_U = 0;
  S.off_V = align_up(make_layout(u.d, u.n, u.m, u.k).total, 256);
  S.off_Z1 = S.off_V + align_up(make_layout(v.d, v.n, v.m, v.k).total, 256);
  S.off_dZ2 = S.off_Z1 + align_up((size_t)v.d * v.m * sizeof(float), 256);
  S.total = S.off_dZ2 + align_up((size_t)u.d * u.m * sizeof(float), 256);
  return S;
}

}  // namespace fasth

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------

using namespace fasth;

extern "C" {

const char* fasth_strerror(int code) {
  switch (code) {
    case FASTH_OK: return "success";
    case FASTH_EINVAL: return "invalid argument (null pointer, non-positive size, or k does not divide n)";
    case FASTH_EWORKSPACE: return "workspace too small";
    case FASTH_EALIGN: return "pointer is not 16-byte aligned";
    case FASTH_EHIP: return "HIP runtime call or kernel launch failed";
    case FASTH_EUNSUPPORTED: return "shape outside the supported range";
    default: return "unknown error code";
  }
}

const char* fasth_kernel_name(int id) {
  switch (id) {
    case FASTH_KERNEL_GRAM: return "gram_partial_kernel";
    case FASTH_KERNEL_TBUILD: return "t_build_kernel";
    case FASTH_KERNEL_CHAIN: return "chain_kernel";
    case FASTH_KERNEL_DV: return "dv_kernel";
    case FASTH_KERNEL_SEQ_FORWARD: return "seq_forward_kernel";
    case FASTH_KERNEL_SEQ_BACKWARD: return "seq_backward_kernel";
    case FASTH_KERNEL_SEQ_REDUCE: return "seq_reduce_kernel";
    case FASTH_KERNEL_DSIGMA: return "dsigma_kernel";
    case FASTH_KERNEL_FACTOR: return "factor_fused_kernel";
    default: return "unknown";
  }
}

int fasth_profile_enable(int on) {
  prof::enabled = on != 0;
  return FASTH_OK;
}

int fasth_profile_collect(float* ms, int* launches) {
  if (!ms || !launches) return FASTH_EINVAL;
  for (int i = 0; i < FASTH_KERNEL_COUNT; ++i) { ms[i] = 0.f; launches[i] = 0; }
  int rc = FASTH_OK;
  for (const prof::Rec& r : prof::recs) {
    float t = 0.f;
    if (r.beg && r.end && hipEventSynchronize(r.end) == hipSuccess &&
        hipEventElapsedTime(&t, r.beg, r.end) == hipSuccess && r.id >= 0 && r.id < FASTH_KERNEL_COUNT) {
      ms[r.id] += t;
      launches[r.id] += 1;
    } else {
      rc = FASTH_EHIP;
    }
    if (r.beg) prof::pool.push_back(r.beg);
    if (r.end) prof::pool.push_back(r.end);
  }
  prof::recs.clear();
  return rc;
}

size_t fasth_workspace_bytes(const fasth_shape* shape) {
  if (check_shape(shape) != FASTH_OK) return 0;
  return make_layout(shape->d, shape->n, shape->m, shape->k).total;
}

int fasth_forward(const fasth_shape* shape, const float* V, const float* X, float* A, void* workspace,
                  size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !X || !A || !workspace) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(X) || !aligned16(A) || !aligned16(workspace)) return FASTH_EALIGN;
  const Product P = bind(shape->d, shape->n, shape->m, shape->k, workspace);
  if (workspace_bytes < P.L.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = build_factors(P, V, st)) != FASTH_OK) return rc;
  return run_chain(P, V, X, A, shape->transpose, true, nullptr, 0, st);
}

int fasth_prepare(const fasth_shape* shape, const float* V, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !workspace) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(workspace)) return FASTH_EALIGN;
  const Product P = bind(shape->d, shape->n, shape->m, shape->k, workspace);
  if (workspace_bytes < P.L.total) return FASTH_EWORKSPACE;
  return build_factors(P, V, static_cast<hipStream_t>(stream));
}

int fasth_apply(const fasth_shape* shape, const float* V, const float* X, float* A, void* workspace,
                size_t workspace_bytes, int save_for_backward, void* stream) {
  int rc = check_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !X || !A || !workspace) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(X) || !aligned16(A) || !aligned16(workspace)) return FASTH_EALIGN;
  const Product P = bind(shape->d, shape->n, shape->m, shape->k, workspace);
  if (workspace_bytes < P.L.total) return FASTH_EWORKSPACE;
  return run_chain(P, V, X, A, shape->transpose, true, nullptr, 0, static_cast<hipStream_t>(stream),
                   save_for_backward != 0);
}

int fasth_backward(const fasth_shape* shape, const float* V, const float* G, float* dV, float* dX, void* workspace,
                   size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !G || !dV || !dX || !workspace) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(G) || !aligned16(dV) || !aligned16(dX) || !aligned16(workspace)) return FASTH_EALIGN;
  const Product P = bind(shape->d, shape->n, shape->m, shape->k, workspace);
  if (workspace_bytes < P.L.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = run_chain(P, V, G, dX, !shape->transpose, false, nullptr, 0, st)) != FASTH_OK) return rc;
  return run_dv(P, V, dV, shape->transpose, st);
}

int fasth_tune_block_size(const fasth_shape* shape, const int* candidates, int ncandidates, int repetitions,
                          const float* V, const float* X, const float* G, float* A, float* dV, float* dX,
                          void* workspace, size_t workspace_bytes, int* best_k, float* best_ms, void* stream) {
  if (!shape || !best_k) return FASTH_EINVAL;
  if (shape->d < 1 || shape->n < 1 || shape->m < 1 || repetitions < 1) return FASTH_EINVAL;
  if ((candidates && ncandidates < 1) || (shape->transpose != 0 && shape->transpose != 1)) return FASTH_EINVAL;
  if (!V || !X || !G || !A || !dV || !dX || !workspace) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(X) || !aligned16(G) || !aligned16(A) || !aligned16(dV) || !aligned16(dX) ||
      !aligned16(workspace))
    return FASTH_EALIGN;
  std::vector<int> ks;
  if (candidates) {
    ks.assign(candidates, candidates + ncandidates);
  } else {
    for (int k = 2; k <= kMaxBlock && k <= shape->n; ++k)
      if (shape->n % k == 0) ks.push_back(k);
    if (ks.empty()) ks.push_back(1);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  FASTH_HIP(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return FASTH_EHIP; }
  int rc = FASTH_OK, found = 0;
  float best = 0.f;
  for (int k : ks) {
    fasth_shape s = *shape;
    s.k = k;
    if (check_shape(&s) != FASTH_OK || fasth_workspace_bytes(&s) > workspace_bytes) continue;  // not a usable candidate
    // one untimed pass, then `repetitions` timed ones
    for (int pass = 0; pass < 2 && rc == FASTH_OK; ++pass) {
      const int reps = pass == 0 ? 1 : repetitions;
      if (pass == 1 && hipEventRecord(e0, st) != hipSuccess) { rc = FASTH_EHIP; break; }
      for (int r = 0; r < reps && rc == FASTH_OK; ++r) {
        rc = fasth_forward(&s, V, X, A, workspace, workspace_bytes, stream);
        if (rc == FASTH_OK) rc = fasth_backward(&s, V, G, dV, dX, workspace, workspace_bytes, stream);
      }
      if (pass == 1 && rc == FASTH_OK) {
        float ms = 0.f;
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
          rc = FASTH_EHIP;
          break;
        }
        ms /= repetitions;
        if (!found || ms < best) { best = ms; *best_k = k; found = 1; }
      }
    }
    if (rc != FASTH_OK) break;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != FASTH_OK) return rc;
  if (!found) return FASTH_EUNSUPPORTED;
  if (best_ms) *best_ms = best;
  return FASTH_OK;
}

size_t fasth_sequential_workspace_bytes(const fasth_shape* shape) {
  if (!shape || shape->d < 1 || shape->n < 1 || shape->m < 1) return 0;
  if (shape->d > kMaxD || shape->m > 65535) return 0;
  return (size_t)shape->m * shape->n * shape->d * sizeof(float) + (size_t)shape->d * shape->m * sizeof(float);
}

static int check_seq_shape(const fasth_shape* s) {
  if (!s) return FASTH_EINVAL;
  if (s->d < 1 || s->n < 1 || s->m < 1) return FASTH_EINVAL;
  if (s->transpose != 0 && s->transpose != 1) return FASTH_EINVAL;
  if (s->d > kMaxD || s->m > 65535) return FASTH_EUNSUPPORTED;
  return FASTH_OK;
}

#define FASTH_SEQ_DISPATCH(KERNEL, per, grid, block, stream, ...)                         \
  do {                                                                                    \
    if ((per) <= 1) hipLaunchKernelGGL(KERNEL<1>, grid, block, 0, stream, __VA_ARGS__);      \
    else if ((per) <= 2) hipLaunchKernelGGL(KERNEL<2>, grid, block, 0, stream, __VA_ARGS__); \
    else if ((per) <= 4) hipLaunchKernelGGL(KERNEL<4>, grid, block, 0, stream, __VA_ARGS__); \
    else if ((per) <= 8) hipLaunchKernelGGL(KERNEL<8>, grid, block, 0, stream, __VA_ARGS__); \
    else hipLaunchKernelGGL(KERNEL<16>, grid, block, 0, stream, __VA_ARGS__);                \
  } while (0)

int fasth_sequential_forward(const fasth_shape* shape, const float* V, const float* X, float* A, void* stream) {
  int rc = check_seq_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !X || !A) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(X) || !aligned16(A)) return FASTH_EALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int threads = seq_threads(shape->d), per = (shape->d + threads - 1) / threads;
  {
    prof::Scope ps_(FASTH_KERNEL_SEQ_FORWARD, st);
    FASTH_SEQ_DISPATCH(seq_forward_kernel, per, dim3(shape->m), dim3(threads), st, V, X, A, shape->d, shape->n,
                       shape->m, shape->transpose);
  }
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

int fasth_sequential_backward(const fasth_shape* shape, const float* V, const float* X, const float* G, float* dV,
                              float* dX, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_seq_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !X || !G || !dV || !dX || !workspace) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(X) || !aligned16(G) || !aligned16(dV) || !aligned16(dX) || !aligned16(workspace))
    return FASTH_EALIGN;
  if (workspace_bytes < fasth_sequential_workspace_bytes(shape)) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int d = shape->d, n = shape->n, m = shape->m;
  float* dVpart = static_cast<float*>(workspace);
  float* A = dVpart + (size_t)m * n * d;
  const int threads = seq_threads(d), per = (d + threads - 1) / threads;
  {
    prof::Scope ps_(FASTH_KERNEL_SEQ_FORWARD, st);
    FASTH_SEQ_DISPATCH(seq_forward_kernel, per, dim3(m), dim3(threads), st, V, X, A, d, n, m, shape->transpose);
  }
  FASTH_HIP(hipGetLastError());
  {
    prof::Scope ps_(FASTH_KERNEL_SEQ_BACKWARD, st);
    FASTH_SEQ_DISPATCH(seq_backward_kernel, per, dim3(m), dim3(threads), st, V, (const float*)A, G, dVpart, dX, d, n,
                       m, shape->transpose);
  }
  FASTH_HIP(hipGetLastError());
  const size_t nd = (size_t)n * d;
  {
    prof::Scope ps_(FASTH_KERNEL_SEQ_REDUCE, st);
    hipLaunchKernelGGL(seq_reduce_kernel, dim3((unsigned)((nd + 255) / 256)), dim3(256), 0, st, (const float*)dVpart,
                       dV, nd, m);
  }
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

size_t svd_layer_workspace_bytes(const fasth_svd_shape* shape) {
  fasth_shape fs;
  if (check_svd_shape(shape, &fs) != FASTH_OK) return 0;
  return make_svd_layout(fs.d, fs.n, fs.m, fs.k).total;
}

int svd_sym_apply(const fasth_svd_shape* shape, int function, const float* Uv, const float* sigma, const float* X,
                  float* Y, void* workspace, size_t workspace_bytes, void* stream) {
  fasth_shape fs;
  int rc = check_svd_shape(shape, &fs);
  if (rc != FASTH_OK) return rc;
  const int mode = sym_scale_mode(function);
  if (mode < 0 || !Uv || !sigma || !X || !Y || !workspace) return FASTH_EINVAL;
  if (!aligned16(Uv) || !aligned16(sigma) || !aligned16(X) || !aligned16(Y) || !aligned16(workspace)) return FASTH_EALIGN;
  const SvdLayout S = make_svd_layout(fs.d, fs.n, fs.m, fs.k);
  if (workspace_bytes < S.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const Product Pin = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_V);   // U^T X; owns the factors
  const Product Pout = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_U);  // U (s * Z1); saves only
  float* Z1 = reinterpret_cast<float*>(ws + S.off_Z1);
  if ((rc = build_factors(Pin, Uv, st)) != FASTH_OK) return rc;
  if ((rc = run_chain(Pin, Uv, X, Z1, 1, true, nullptr, 0, st)) != FASTH_OK) return rc;
  return run_chain(Pout, Uv, Z1, Y, 0, true, sigma, mode, st, true, Pin.T());
}

int svd_sym_apply_backward(const fasth_svd_shape* shape, int function, const float* Uv, const float* sigma,
                           const float* G, float* dUv, float* dsigma, float* dX, void* workspace,
                           size_t workspace_bytes, void* stream) {
  fasth_shape fs;
  int rc = check_svd_shape(shape, &fs);
  if (rc != FASTH_OK) return rc;
  const int mode = sym_scale_mode(function);
  if (mode < 0 || !Uv || !sigma || !G || !dUv || !dsigma || !dX || !workspace) return FASTH_EINVAL;
  if (!aligned16(Uv) || !aligned16(sigma) || !aligned16(G) || !aligned16(dUv) || !aligned16(dsigma) ||
      !aligned16(dX) || !aligned16(workspace))
    return FASTH_EALIGN;
  const SvdLayout S = make_svd_layout(fs.d, fs.n, fs.m, fs.k);
  if (workspace_bytes < S.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const Product Pin = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_V);
  const Product Pout = bind(fs.d, fs.n, fs.m, fs.k, ws + S.off_U);
  const float* Z1 = reinterpret_cast<const float*>(ws + S.off_Z1);
  float* dZ2 = reinterpret_cast<float*>(ws + S.off_dZ2);
  if ((rc = run_chain(Pout, Uv, G, dZ2, 1, false, nullptr, 0, st, true, Pin.T())) != FASTH_OK) return rc;
  if ((rc = run_dv(Pout, Uv, dUv, 0, st)) != FASTH_OK) return rc;
  if ((rc = run_chain(Pin, Uv, dZ2, dX, 0, false, sigma, mode, st, true, nullptr, -1, Z1, dsigma, fs.d)) != FASTH_OK)
    return rc;
  return run_dv(Pin, Uv, dUv, 1, st, true);
}

int svd_layer_log_abs_det(int d, const float* sigma, float* log_abs_det, float* dsigma, void* stream) {
  if (d < 1 || !sigma || !log_abs_det) return FASTH_EINVAL;
  if (!aligned16(sigma) || (dsigma && !aligned16(dsigma))) return FASTH_EALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(logabsdet_kernel, dim3(1), dim3(256), 0, st, sigma, log_abs_det, dsigma, d);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

int svd_layer_apply(const fasth_svd_shape* shape, const float* Uv, const float* sigma, const float* Vv, const float* X,
                    float* Y, void* workspace, size_t workspace_bytes, void* stream) {
  return svd_forward(shape, Vv, sigma, Uv, X, Y, workspace, workspace_bytes, stream, 1);
}

int svd_layer_inverse_apply(const fasth_svd_shape* shape, const float* Uv, const float* sigma, const float* Vv,
                            const float* X, float* Y, void* workspace, size_t workspace_bytes, void* stream) {
  return svd_forward(shape, Uv, sigma, Vv, X, Y, workspace, workspace_bytes, stream, 2);
}

int svd_layer_apply_backward(const fasth_svd_shape* shape, const float* Uv, const float* sigma, const float* Vv,
                             const float* G, float* dUv, float* dsigma, float* dVv, float* dX, void* workspace,
                             size_t workspace_bytes, void* stream) {
  return svd_backward(shape, Vv, sigma, Uv, G, dVv, dsigma, dUv, dX, workspace, workspace_bytes, stream, 1);
}

int svd_layer_inverse_apply_backward(const fasth_svd_shape* shape, const float* Uv, const float* sigma,
                                     const float* Vv, const float* G, float* dUv, float* dsigma, float* dVv,
                                     float* dX, void* workspace, size_t workspace_bytes, void* stream) {
  return svd_backward(shape, Uv, sigma, Vv, G, dUv, dsigma, dVv, dX, workspace, workspace_bytes, stream, 2);
}

size_t svd_rect_workspace_bytes(const fasth_rect_shape* shape) {
  fasth_shape fu, fv;
  if (check_rect_shape(shape, &fu, &fv) != FASTH_OK) return 0;
  return make_rect_layout(fu, fv).total;
}

int svd_rect_apply(const fasth_rect_shape* shape, const float* Uv, const float* sigma, const float* Vv, const float* X,
                   float* Y, void* workspace, size_t workspace_bytes, void* stream) {
  fasth_shape fu, fv;
  int rc = check_rect_shape(shape, &fu, &fv);
  if (rc != FASTH_OK) return rc;
  if (!Uv || !sigma || !Vv || !X || !Y || !workspace) return FASTH_EINVAL;
  if (!aligned16(Uv) || !aligned16(sigma) || !aligned16(Vv) || !aligned16(X) || !aligned16(Y) || !aligned16(workspace))
    return FASTH_EALIGN;
  const RectLayout S = make_rect_layout(fu, fv);
  if (workspace_bytes < S.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const Product Pu = bind(fu.d, fu.n, fu.m, fu.k, ws + S.off_U);
  const Product Pv = bind(fv.d, fv.n, fv.m, fv.k, ws + S.off_V);
  float* Z1 = reinterpret_cast<float*>(ws + S.off_Z1);
  const int r = fu.d < fv.d ? fu.d : fv.d;
  if ((rc = build_factors_pair(Pv, Vv, Pu, Uv, st)) != FASTH_OK) return rc;
  if ((rc = run_chain(Pv, Vv, X, Z1, 1, true, nullptr, 0, st)) != FASTH_OK) return rc;
  // Sigma Z1: the first r rows of Z1 scaled by sigma, rows r..rows-1 zero; fused into the chain's load
  return run_chain(Pu, Uv, Z1, Y, 0, true, sigma, 1, st, true, nullptr, r);
}

int svd_rect_apply_backward(const fasth_rect_shape* shape, const float* Uv, const float* sigma, const float* Vv,
                            const float* G, float* dUv, float* dsigma, float* dVv, float* dX, void* workspace,
                            size_t workspace_bytes, void* stream) {
  fasth_shape fu, fv;
  int rc = check_rect_shape(shape, &fu, &fv);
  if (rc != FASTH_OK) return rc;
  if (!Uv || !sigma || !Vv || !G || !dUv || !dsigma || !dVv || !dX || !workspace) return FASTH_EINVAL;
  if (!aligned16(Uv) || !aligned16(sigma) || !aligned16(Vv) || !aligned16(G) || !aligned16(dUv) ||
      !aligned16(dsigma) || !aligned16(dVv) || !aligned16(dX) || !aligned16(workspace))
    return FASTH_EALIGN;
  const RectLayout S = make_rect_layout(fu, fv);
  if (workspace_bytes < S.total) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const Product Pu = bind(fu.d, fu.n, fu.m, fu.k, ws + S.off_U);
  const Product Pv = bind(fv.d, fv.n, fv.m, fv.k, ws + S.off_V);
  const float* Z1 = reinterpret_cast<const float*>(ws + S.off_Z1);
  float* dZ2 = reinterpret_cast<float*>(ws + S.off_dZ2);
  const int r = fu.d < fv.d ? fu.d : fv.d;
  if ((rc = run_chain(Pu, Uv, G, dZ2, 1, false, nullptr, 0, st)) != FASTH_OK) return rc;
  // Sigma^T dZ2: first r rows scaled, rows r..cols-1 zero
  if ((rc = run_chain(Pv, Vv, dZ2, dX, 0, false, sigma, 1, st, true, nullptr, r, Z1, dsigma, r)) != FASTH_OK) return rc;
  return run_dv_pair(Pu, Uv, dUv, 0, Pv, Vv, dVv, 1, st);
}

}  // extern "C"
