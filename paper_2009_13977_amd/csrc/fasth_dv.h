// Algorithm 2 Step 2: the gradients of the Householder vectors as dense products per block (dv_kernel, dv_z_kernel).
// Included by fasth.hip, the library's single translation unit.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

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
  float* dVpart;        // [msplit][n][d]: partial sums when the mini-batch is split over workgroups
  int msplit;           // workgroups per (tile, block) along the mini-batch; 1: no split
  int cols_per_part;    // columns per such workgroup, a multiple of the chunk of 32 (m rounded up if msplit = 1)
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
  // blockIdx.z = product * msplit + part of the mini-batch (msplit is the same for both products of a launch)
  // (a launch has at most two products, so the product index needs no division)
  const int msplit = pair.a[0].msplit, which = (int)blockIdx.z >= msplit ? 1 : 0, part = (int)blockIdx.z - which * msplit;
  const DvArgs p = pair.a[which];
  const int k = p.k, d = p.d, m = p.m, n = p.n;
  if ((int)blockIdx.y * k >= n || (int)blockIdx.x * kDvTile >= d) return;  // whole workgroup, before any barrier
  // this workgroup's columns: whole chunks of kDvMChunk (cols_per_part comes from the host)
  const int m_begin = part * p.cols_per_part, m_end = min(m, m_begin + p.cols_per_part);
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
  fetch(m_begin < m ? m_begin : 0, cur);
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
  for (int mc = m_begin; mc < m_end; mc += kDvMChunk) {
    if (mc > m_begin) __syncthreads();
    to_lds(cur);
    __syncthreads();
    if (mc + kDvMChunk < m_end) fetch(mc + kDvMChunk, cur);  // in flight during this chunk's products
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
      if (part == 0) ev = tile_mma_rows<kp>(Es + ti * 16 * LDE, LDE, Vs + tx * 16, LDX, ev);  // E V_i enters once
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int j = ti * 16 + 4 * q + jj, x = x0 + tx * 16 + li;
        if (j < k && x < d) {
          const float val = ev[jj] - acc[w][jj];
          if (msplit > 1) {
            p.dVpart[((size_t)part * n + (size_t)i * k + j) * d + x] = val;  // summed by dv_sum_kernel
          } else {
            float* dst = p.dV + ((size_t)i * k + j) * d + x;
            *dst = p.accumulate ? *dst + val : val;
          }
        }
      }
    }
  }
}

// dV = sum of the mini-batch parts (fixed order), for up to two products: blockIdx.y picks the product.
__global__ void __launch_bounds__(256) dv_sum_kernel(DvPair pair) {
  const DvArgs p = pair.a[blockIdx.y];
  const size_t nd = (size_t)p.n * p.d, idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= nd) return;
  float sum = p.dVpart[idx];
  for (int part = 1; part < p.msplit; ++part) sum += p.dVpart[(size_t)part * nd + idx];
  p.dV[idx] = p.accumulate ? p.dV[idx] + sum : sum;
}

static size_t dv_lds(int kp) {
  return sizeof(float) * ((size_t)kp * (kp + 4) + 2 * (size_t)kp * (kDvMChunk + 4) +
                          2 * (size_t)kDvMChunk * (kDvTile + 4) + (size_t)kp * (kDvTile + 4));
}

}  // namespace fasth
