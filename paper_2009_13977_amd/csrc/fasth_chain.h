// Algorithm 1 Step 2 and Algorithm 2 Step 1: the sequential block chain (chain_pipe_kernel, chain_tile_kernel,
// chain_kernel) and its launcher.
// Included by fasth.hip, the library's single translation unit.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// The sequential block chain (Algorithm 1 Step 2; Algorithm 2 Step 1, Eq. 3).
// One workgroup per column of the d x m input: columns never interact, so no workgroup waits for
// another. Per block i:  B = V_i a,  C = op(T_i) B,  a <- a - V_i^T C,
// op(T) = T for P_i (blocks nb..1), T^T for P_i^T (blocks 1..nb).
// The k inner products of a block are independent, which is the parallelism FastH adds over the
// one-at-a-time algorithm.
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
  const float* Tt;        // [nb][kp][kp]: the transposed factors
  const float* in;        // [d][m]
  float* out;             // [d][m]
  float* save_in;         // [nb][m][d] or null
  float* save_c;          // [m][n] or null
  const float* in_scale;  // [d] or null: input row x is multiplied by diag_factor(in_scale_mode, in_scale[x])
  int in_scale_mode;
  int in_rows;            // rows of `in` that exist; rows in_rows..d-1 of the chain's input are zero
  int d, n, m, k, kp, nb;
  int transpose;
  int sub;                // chain_pipe_kernel, chain_quad_kernel, chain_team_tile_kernel: steps per block (set by their launchers)
  // Optional side product of the SVD layers' backward pass, which has the chain's input as one operand:
  // ds_out[r] = s'(in_scale[r]) sum_l in[r][l] ds_z1[r][l] for r < ds_rows (s = diag_factor(in_scale_mode, .)).
  // Null ds_out: not wanted. Kernels that cannot take it along leave it to a launch of dsigma_kernel.
  const float* ds_z1;     // [ds_rows][m]
  float* ds_out;          // [ds_rows]
  int ds_rows;
  // Hand-off area of the workspace for kernels in which workgroups share a column (null: the shape has none), and
  // the number of polls after which a wait for another workgroup gives up.
  unsigned* xch;
  int wait_limit;
  int parts;              // chain_team_kernel: workgroups per column (set by its launcher)
  const float* S;         // chain_team_wide_kernel: [n / 128][2][64][64], V_a V_b^T of each step's two blocks and its transpose
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

// General form for vectors too long for the register-resident kernels: 1024 threads, thread t owns the chunks of
// four consecutive elements x = 4 (t + 1024 u) .. + 3, u < U, so a wave fetches 1 KiB of a row at a time. A block's
// rows pass through the registers twice, once per product (the second time from the cache). Rows are fetched
// through a buffer descriptor spanning the block, so any d works: 4-byte alignment is enough for it, what lies
// beyond the block reads as zero, and elements of a row's last chunk that hang over the row's end are masked.
template <int U>
__global__ void __launch_bounds__(1024) chain_kernel(ChainArgs p) {
  extern __shared__ float smem[];
  constexpr int NT = 1024, NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = blockIdx.x;
  const int d = p.d, k = p.k, kp = p.kp, m = p.m;
  const int LDT = kp + 1;
  float* Ts = smem;               // [kp][LDT]
  float* Bpart = Ts + kp * LDT;   // [NW][kp]
  float* Bv = Bpart + NW * kp;    // [kp]
  float* Cv = Bv + kp;            // [kp]
  float a[U][4];
  unsigned off[U];  // byte offset of chunk u within a row, or beyond every buffer if the chunk does not exist
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int x0 = 4 * (tid + u * NT);
    off[u] = x0 < d ? (unsigned)x0 * 4u : kOob;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int x = x0 + r;
      float v = 0.f;
      if (x < d && x < p.in_rows) {
        v = p.in[(size_t)x * m + col];
        if (p.in_scale_mode) v *= diag_factor(p.in_scale_mode, p.in_scale[x]);
      }
      a[u][r] = v;
    }
  }
  const int sel = reduce_sel<8>(lane);
  for (int s = 0; s < p.nb; ++s) {
    const int i = p.transpose ? s : p.nb - 1 - s;
    const BufferDesc vdesc = make_buffer(p.V + (size_t)i * k * d, (size_t)k * d * sizeof(float));
    const float* Ti = p.T + (size_t)i * kp * kp;
    for (int idx = tid; idx < kp * kp; idx += NT) Ts[(idx / kp) * LDT + idx % kp] = Ti[idx];
    if (p.save_in) {
      float* dst = p.save_in + ((size_t)i * m + col) * d;
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int x = 4 * (tid + u * NT) + r;
          if (x < d) dst[x] = a[u][r];
        }
      }
    }
    for (int j0 = 0; j0 < k; j0 += 8) {
      float pj[8];
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        pj[jj] = 0.f;
        // rows past the block lie beyond the buffer and read as zero
        const unsigned row_off = (unsigned)(j0 + jj) * (unsigned)d * 4u;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const BufVec<4> v = buffer_load<4>(vdesc, off[u], row_off);
#pragma unroll
          for (int r = 0; r < 4; ++r) pj[jj] = fmaf(v.e[r], a[u][r], pj[jj]);  // a is zero where the chunk hangs over
        }
      }
      wave_reduce_multi<8>(pj);
      if ((lane & reduce_writer_mask<8>()) == 0 && j0 + sel < kp) Bpart[wave * kp + j0 + sel] = pj[0];
    }
    __syncthreads();
    if (tid < kp) {
      float b = 0.f;
      if (tid < k)
        for (int w = 0; w < NW; ++w) b += Bpart[w * kp + tid];
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
      const unsigned row_off = (unsigned)j * (unsigned)d * 4u;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const BufVec<4> v = buffer_load<4>(vdesc, off[u], row_off);
#pragma unroll
        for (int r = 0; r < 4; ++r) a[u][r] = fmaf(-c, v.e[r], a[u][r]);
      }
    }
    // elements beyond d have just seen the next row's values: back to zero
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (4 * (tid + u * NT) + r >= d) a[u][r] = 0.f;
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int x = 4 * (tid + u * NT) + r;
      if (x < d) p.out[(size_t)x * m + col] = a[u][r];
    }
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
// RL: rows of the next block fetched during the reduction; P1: during the first product (0: half of the rest);
// XB: at each of four points next to the two barriers (before and after each), where a wave waits anyway: for the
// other waves, or for the LDS reads it has just issued. A fetch keeps the issuing wave from its arithmetic for ~35
// clocks, so the fewer of them sit between the multiply-adds the better (d = 4096: 1.61 -> 1.40 ms per forward +
// backward with XB = 1, d = 2048: 396 -> 372 us, d = 1024: 113.7 -> 112.2 us).
// UNAL: d is not a multiple of VW, so rows are not 16-byte aligned and the last chunk of a row hangs over its end.
// Rows are then fetched through a buffer that spans the block (4-byte alignment is enough for it, and what lies
// beyond the block reads as zero); the overhanging elements see the next row's values, so they are put back to
// zero after every update and never stored.
template <int K, int VW, int NT, int RL = 0, int SUB = 1, bool PAD = false, int P1 = 0, bool UNAL = false, int XB = 0>
__global__ void __launch_bounds__(NT) chain_pipe_kernel(ChainArgs p) {
  typedef PipeRegs<K, VW, NT> Regs;
  constexpr int NW = NT / 64, G = Regs::G, LPT = Regs::LPT;
  constexpr int PR = P1 > 0 ? P1 : (K - RL) / 2;  // rows of the next block fetched during the first product
  constexpr int PR2 = K - RL - PR - 4 * XB;         // ... and during the second
  constexpr int X0 = PR + RL;                       // first of the 4 XB rows fetched on either side of the two barriers
  constexpr int S1 = K / PR, S2 = K / PR2;          // one fetch every S1 (S2) rows of the product
  static_assert(PR >= 1 && PR2 >= 1 && S1 >= 1 && S2 >= 1, "prefetch split");
  static_assert(K % 4 == 0 && K * G <= NT && LPT >= 1, "shape");
  static_assert(RL % 2 == 0 && RL <= K / 4 && (RL == 0 || K >= 8), "prefetch split");
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
  bool keep[VW];  // elements of this thread's chunk that exist
#pragma unroll
  for (int r = 0; r < VW; ++r) keep[r] = ok && (!UNAL || x0 + r < (unsigned)d);
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
  auto load_row = [&](int i, int j) {
    if constexpr (UNAL) {
      // the buffer spans the step's block of k rows (at most 2 MiB), so V itself may be of any size
      const BufferDesc vdesc = make_buffer(p.V + (size_t)step_block(i) * p.k * d, (size_t)p.k * d * sizeof(float));
      const unsigned row = (unsigned)(step_part(i) * K + (PAD ? min(j, rows_valid(i) - 1) : j));
      const BufVec<VW> v = buffer_load<VW>(vdesc, x0 * 4u, row * (unsigned)d * 4u);
      Chunk<VW> c;
#pragma unroll
      for (int r = 0; r < VW; ++r) c.e[r] = v.e[r];
      return c;
    } else {
      return load_chunk<VW>(row_ptr(i, j));
    }
  };
  auto load_t = [&](int i, Regs& r) {
    const int LDT = (SUB > 0 && !PAD && K * SUB >= 16) ? K * SUB : p.kp;  // row stride of the stored factor
    // rows of op(T): of the factor itself or of its stored transpose, so a thread's LPT entries are consecutive in
    // memory either way (one 16-byte fetch for every four) as its partial sums are in LDS
    const float* Ti = (p.transpose ? p.Tt : p.T) + (size_t)step_block(i) * LDT * LDT + (size_t)step_part(i) * (K * LDT + K);
    const float* src = Ti + (t_active ? trow : 0) * LDT + tg * LPT;
    if constexpr (LPT % 4 == 0) {
#pragma unroll
      for (int e4 = 0; e4 < LPT / 4; ++e4) {
        const float4 t4 = reinterpret_cast<const float4*>(src)[e4];
        r.t[4 * e4] = t4.x; r.t[4 * e4 + 1] = t4.y; r.t[4 * e4 + 2] = t4.z; r.t[4 * e4 + 3] = t4.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < LPT; ++e) r.t[e] = src[e];
    }
  };

  // Applies block i held in `cur` while fetching block inext into `nxt`.
  auto apply_block = [&](int i, Regs& cur, int inext, Regs& nxt) {
    if (p.save_in && ok && (SUB == 1 || step_part(i) == (p.transpose ? 0 : sub - 1))) {
      float* dst = p.save_in + ((size_t)step_block(i) * m + col) * d + x0;
      if constexpr (UNAL) {
#pragma unroll
        for (int r = 0; r < VW; ++r)
          if (keep[r]) dst[r] = a.e[r];
      } else {
        store_chunk<VW>(dst, a);
      }
    }
    const int kv = rows_valid(i);
    float pj[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
      if (j % S1 == 0 && j / S1 < PR) {
        nxt.v[j / S1] = load_row(inext, j / S1);
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
          nxt.v[PR + t / 4] = load_row(inext, PR + t / 4);
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      wave_reduce_multi_reg<K>(pj, prefetch);
    } else {
      wave_reduce_multi_reg<K>(pj);
    }
    if ((lane & reduce_writer_mask<K>()) == 0) Bpart[wave][sel] = pj[0];
    auto fetch_at_barrier = [&](int q) {
#pragma unroll
      for (int e = 0; e < XB; ++e) nxt.v[X0 + q * XB + e] = load_row(inext, X0 + q * XB + e);
      if constexpr (XB > 0) __builtin_amdgcn_sched_barrier(0);
    };
    fetch_at_barrier(0);
    lds_barrier();
    fetch_at_barrier(1);
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
    fetch_at_barrier(2);
    lds_barrier();
    fetch_at_barrier(3);
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
        nxt.v[X0 + 4 * XB + j / S2] = load_row(inext, X0 + 4 * XB + j / S2);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int r = 0; r < VW; ++r) a.e[r] = fmaf(-cc[(j / CG) & 1][j % CG], cur.v[j].e[r], a.e[r]);
    }
#pragma unroll
    for (int r = 0; r < VW; ++r)
      if (!keep[r]) a.e[r] = 0.f;
  };

  Regs ra, rb;
#pragma unroll
  for (int j = 0; j < K; ++j) ra.v[j] = load_row(block_of(0), j);
  load_t(block_of(0), ra);
  int s = 0;
  for (; s + 1 < nb; s += 2) {
    apply_block(block_of(s), ra, block_of(s + 1), rb);
    apply_block(block_of(s + 1), rb, block_of(s + 2 < nb ? s + 2 : s + 1), ra);
  }
  if (s < nb) apply_block(block_of(s), ra, block_of(s), rb);
#pragma unroll
  for (int r = 0; r < VW; ++r)
    if (keep[r]) p.out[(size_t)(x0 + r) * m + col] = a.e[r];
}

template <int K, int VW, int NT, int RL = 0, int SUB = 1, bool PAD = false, int P1 = 0, bool UNAL = false, int XB = 0>
static int launch_chain_pipe(const ChainArgs& args, hipStream_t stream) {
  ChainArgs a = args;
  a.sub = SUB > 0 ? SUB : (args.k + K - 1) / K;
  a.nb = args.nb * a.sub;
  if ((size_t)VW * NT < (size_t)a.d || (PAD ? (a.sub * K > a.kp || a.sub != (a.k + K - 1) / K) : a.sub * K != a.k) ||
      (!UNAL && a.d % VW != 0))
    return FASTH_EINVAL;
  const int side = a.ds_out ? (a.ds_rows + NT / 64 - 1) / (NT / 64) : 0;
  static const std::string name = variant_name("chain_pipe_kernel", {K, VW, NT, RL, SUB, PAD, P1, UNAL, XB});
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, name.c_str());
  hipLaunchKernelGGL((chain_pipe_kernel<K, VW, NT, RL, SUB, PAD, P1, UNAL, XB>), dim3(a.m + side), dim3(NT), 0, stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

}  // namespace fasth

#include "fasth_chain_tile.h"  // chain_tile_kernel: the same steps on the matrix cores, for wide mini-batches
#include "fasth_chain_pair.h"  // chain_pair_kernel: the per-column chain with two waves per SIMD
#include "fasth_chain_quad.h"  // chain_quad_kernel: four columns per workgroup on the matrix cores, 256 < m <= 1024
#include "fasth_chain_team.h"  // chain_team_kernel, chain_team_wide_kernel: two to eight workgroups per column, steps of 64 or 128 rows, few columns
#include "fasth_chain_teamtile.h"  // chain_team_tile_kernel: 16 columns per two to four workgroups on the matrix cores, some hundred columns

namespace fasth {

// chain_pipe_kernel serves every d up to 4096; it also takes the side product along.
static bool chain_uses_pipe(const ChainArgs& a) {
  return !chain_uses_tile(a) && !chain_uses_quad(a) && !chain_uses_team_tile(a) && !chain_uses_team_wide(a) && !chain_uses_team(a) && !chain_uses_split_pair(a) && a.d <= 4096;
}
static bool chain_takes_side_product(const ChainArgs& a) { return chain_uses_pipe(a) || chain_uses_team(a) || chain_uses_team_wide(a) || chain_uses_team_tile(a); }

static int launch_chain_kernel(const ChainArgs& a, hipStream_t stream) {
  const int d = a.d, k = a.k;
  if (chain_uses_team_tile(a)) return launch_chain_team_tile(a, stream);
  if (chain_uses_tile(a)) return launch_chain_tile(a, stream);
  if (chain_uses_quad(a)) return launch_chain_quad(a, stream);
  if (chain_uses_team_wide(a)) return launch_chain_team_wide(a, stream);
  if (chain_uses_team(a)) return launch_chain_team(a, stream);
  if (chain_uses_split_pair(a)) {
    // two compute units per column, 32-row steps (d = n = 2048, m = 64: see the measurements at the kernel)
    if (k == 32) return launch_chain_split_pair<1>(a, stream);
    if (k == 64) return launch_chain_split_pair<2>(a, stream);
    return launch_chain_split_pair<4>(a, stream);
  }
  if (chain_uses_pipe(a) && d % 4 != 0) {
    // rows not 16-byte aligned: the general form of the kernels (any block size, short last step)
    if (chain_pair_serves(a) && (a.m <= (d > 896 ? 176 : kComputeUnits) || d <= 512)) {  // as for aligned rows below
      if (d <= 256) return launch_chain_pair<2, 0, 4, 4, 3, 2, true, true>(a, stream);
      if (d <= 512) return launch_chain_pair<4, 0, 4, 4, 3, 2, true, true>(a, stream);
      return launch_chain_pair<8, 0, 4, 4, 3, 2, true, true>(a, stream);
    }
    if (d <= 1024) {
      if (k <= 8) return launch_chain_pipe<8, 4, 256, 2, 0, true, 0, true>(a, stream);
      if (k <= 16) return launch_chain_pipe<16, 4, 256, 4, 0, true, 0, true>(a, stream);
      return launch_chain_pipe<32, 4, 256, 8, 0, true, 7, true, 1>(a, stream);
    } else if (d <= 2048) {
      if (k <= 8) return launch_chain_pipe<8, 4, 512, 2, 0, true, 1, true, 1>(a, stream);
      return launch_chain_pipe<16, 4, 512, 4, 0, true, 4, true, 1>(a, stream);
    }
    return launch_chain_pipe<8, 4, 1024, 2, 0, true, 1, true, 1>(a, stream);
  }
  if (chain_uses_pipe(a)) {
    // whole block in registers, two copies; a quarter of the next block is fetched during the reduction
    if (k == 16 && d <= 256) return launch_chain_pipe<16, 1, 256, 4, 1, false, 4, false, 1>(a, stream);  // narrower lanes keep all four waves busy
    if (k == 16 && d <= 512) return launch_chain_pipe<16, 2, 256, 4, 1, false, 4, false, 1>(a, stream);
    if (k == 8 && d <= 256) return launch_chain_pipe<8, 1, 256, 2>(a, stream);
    if (k == 8 && d <= 512) return launch_chain_pipe<8, 2, 256, 2>(a, stream);
    if (k == 16 && d <= 1024) return launch_chain_pipe<16, 4, 256, 4, 1, false, 4, false, 1>(a, stream);
    if (k == 16 && d <= 2048) return launch_chain_pipe<16, 4, 512, 4, 1, false, 4, false, 1>(a, stream);
    // Blocks of 32, 64 or 128 rows, at most one column per compute unit: one wave per 128 elements of the column,
    // pairs of lanes sharing a chunk (d = n = 1024, m = 32, k = 32: 108.6 -> 102.3 us per forward + backward against
    // the kernels below; d = 512: 54.2 -> 44.8 us; d = 256: 30.4 -> 29.1 us)
    // (with more columns than compute units it stays the faster one up to d = 512, where two or four of its workgroups
    // share a unit: d = 512, m = 512: 108 -> 86 us, m = 1024: 194 -> 148 us; beyond, the 16-row steps further down win)
    // (at d = 1024 the 4-wave kernel is the faster one again from about 180 columns on, when most compute units of
    // an XCD stream V from its L2 at once: m = 160: 120.5 -> 118.4 us, m = 192: 121.8 -> 122.6, m = 256: 127.7 -> 133.4;
    // at d = 768 the pairs win up to 256 columns, 101.2 -> 92.7 us)
    const int pair_max_cols = d > 896 ? 176 : kComputeUnits;
    if (chain_pair_serves(a) && (a.m <= pair_max_cols || d <= 512)) {
#define FASTH_LAUNCH_PAIR(NW)                                                             \
  do {                                                                                    \
    if (k == 32) return launch_chain_pair<NW, 1, 4, 4, 3, 2>(a, stream);                  \
    if (k == 64) return launch_chain_pair<NW, 2, 4, 4, 3, 2>(a, stream);                  \
    if (k == 128) return launch_chain_pair<NW, 4, 4, 4, 3, 2>(a, stream);                 \
    if (k < 32) return launch_chain_pair<NW, 1, 4, 4, 3, 2, true>(a, stream);             \
    if (k < 64) return launch_chain_pair<NW, 2, 4, 4, 3, 2, true>(a, stream);             \
    if (k <= 96) return launch_chain_pair<NW, 3, 4, 4, 3, 2, true>(a, stream);            \
    return launch_chain_pair<NW, 4, 4, 4, 3, 2, true>(a, stream);                         \
  } while (0)
      if (d <= 256) FASTH_LAUNCH_PAIR(2);
      if (d <= 512) FASTH_LAUNCH_PAIR(4);
      FASTH_LAUNCH_PAIR(8);
#undef FASTH_LAUNCH_PAIR
    }
    // More columns than compute units (and too few for the matrix-core kernel): steps of 16 rows take 166 registers
    // against the 291 of 32-row steps, so three workgroups share a compute unit and fill each other's waits
    // (d = 1024, k = 32, per forward + backward: m = 384: 233 -> 194 us, m = 512: 244 -> 222, m = 768: 356 -> 321;
    // up to 256 columns the 32-row steps are the faster ones: 137 against 149 us at m = 256).
    if (a.m > kComputeUnits && d > 512 && d <= 1024) {
      if (k == 32) return launch_chain_pipe<16, 4, 256, 4, 2, false, 4, false, 1>(a, stream);
      if (k == 64) return launch_chain_pipe<16, 4, 256, 4, 4, false, 4, false, 1>(a, stream);
      if (k == 128) return launch_chain_pipe<16, 4, 256, 4, 8, false, 4, false, 1>(a, stream);
    }
    // (7 of the 32 rows of the next block fetched during the first product, 8 during the reduction, 4 next to the
    // barriers, 13 during the update)
    if (k == 32 && d <= 1024) return launch_chain_pipe<32, 4, 256, 8, 1, false, 7, false, 1>(a, stream);
    // Larger blocks and longer vectors: two register copies of the whole block do not fit, but the block can be
    // applied as steps of 32 rows (d <= 1024) or 16 rows (d <= 2048, two waves per SIMD), which is faster than
    // one copy refilled in place or rows streamed twice (d = n = 2048: 178 us for k = 32, 64 and 128 alike,
    // against 222, 359 and 406 us)
    if (d <= 1024) {
      if (k == 64) return launch_chain_pipe<32, 4, 256, 8, 2, false, 7, false, 1>(a, stream);
      if (k == 128) return launch_chain_pipe<32, 4, 256, 8, 4, false, 7, false, 1>(a, stream);
      if (k == 8) return launch_chain_pipe<8, 4, 256, 2, 1, false, 1, false, 1>(a, stream);
      // any other block size: steps of 8, 16 or 32 rows, the last one of a block short
      if (k < 8) return launch_chain_pipe<8, 4, 256, 2, 1, true, 1, false, 1>(a, stream);
      if (k < 16) return launch_chain_pipe<16, 4, 256, 4, 1, true, 4, false, 1>(a, stream);
      if (k < 32) return launch_chain_pipe<32, 4, 256, 8, 1, true, 7, false, 1>(a, stream);  // one short step per block
      if (k < 64) return launch_chain_pipe<32, 4, 256, 8, 2, true, 7, false, 1>(a, stream);  // a full step and a short one
      if (k > 96) return launch_chain_pipe<32, 4, 256, 8, 4, true, 7, false, 1>(a, stream);
      return launch_chain_pipe<32, 4, 256, 8, 0, true, 7, false, 1>(a, stream);
    } else if (d <= 2048) {
      if (k == 32) return launch_chain_pipe<16, 4, 512, 4, 2, false, 4, false, 1>(a, stream);  // fetch split 4 / 4 / 4 / 4
      if (k == 64) return launch_chain_pipe<16, 4, 512, 4, 4, false, 4, false, 1>(a, stream);
      if (k == 128) return launch_chain_pipe<16, 4, 512, 4, 8, false, 4, false, 1>(a, stream);
      if (k == 8) return launch_chain_pipe<8, 4, 512, 2, 1, false, 1, false, 1>(a, stream);
      if (k < 8) return launch_chain_pipe<8, 4, 512, 2, 0, true, 1, false, 1>(a, stream);
      return launch_chain_pipe<16, 4, 512, 4, 0, true, 4, false, 1>(a, stream);
    } else {
      // 16 waves share 512 registers per lane: two copies of 8 rows
      if (k % 8 == 0) return launch_chain_pipe<8, 4, 1024, 2, 0, false, 1, false, 1>(a, stream);
      return launch_chain_pipe<8, 4, 1024, 2, 0, true, 1, false, 1>(a, stream);
    }
  }
  // longer vectors: the general kernel
  const int threads = 1024, nw = threads / 64;
  const int per = (d + 4 * threads - 1) / (4 * threads);  // chunks of four elements per thread
  const size_t lds = sizeof(float) * ((size_t)a.kp * (a.kp + 1) + (size_t)nw * a.kp + 2 * a.kp);
  dim3 grid(a.m), block(threads);
#define FASTH_LAUNCH_CHAIN(UU)                                                   \
  do {                                                                           \
    int rc_ = allow_lds(chain_kernel<UU>, lds);                                  \
    if (rc_ != FASTH_OK) return rc_;                                             \
    static const std::string name_ = variant_name("chain_kernel", {UU});         \
    prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, name_.c_str());                  \
    hipLaunchKernelGGL(chain_kernel<UU>, grid, block, lds, stream, a);           \
  } while (0)
  if (per > 4) return FASTH_EUNSUPPORTED;  // d > 16384: check_shape refuses it before
  if (per <= 2) FASTH_LAUNCH_CHAIN(2);
  else if (per == 3) FASTH_LAUNCH_CHAIN(3);
  else FASTH_LAUNCH_CHAIN(4);
#undef FASTH_LAUNCH_CHAIN
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

static int launch_chain(const ChainArgs& a, hipStream_t stream) {
  const int rc = launch_chain_kernel(a, stream);
  if (rc != FASTH_OK || !a.ds_out || chain_takes_side_product(a)) return rc;
  prof::Scope ps_(FASTH_KERNEL_DSIGMA, stream, "dsigma_kernel");
  hipLaunchKernelGGL(dsigma_kernel, dim3((a.ds_rows + 3) / 4), dim3(256), 0, stream, a.in, a.ds_z1, a.in_scale, a.ds_out,
                     a.ds_rows, a.m, a.in_scale_mode);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

}  // namespace fasth
