// Algorithm 1 Step 2 and Algorithm 2 Step 1 on the matrix cores, for mini-batches of many columns (chain_tile_kernel).
// Included by fasth_chain.h after ChainArgs and diag_factor.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

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

// kTileGroups: groups per wave, the same for all waves (a group that lies beyond d is all zeros: its
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
      // A lane holds 64 contiguous bytes of its column per group, as four 16-byte pieces j (x = .. + 4 j). Stored as
      // they lie, the 64 lanes of a store would touch 64 different cache lines (adjacent lanes are adjacent COLUMNS,
      // d floats apart), which costs the address unit four times a coalesced store. So the four lanes of a quad
      // (columns 4a .. 4a + 3) first transpose their 4 x 4 pieces: in store t, lane 4a + b then writes piece b of
      // column 4a + t, and each quad covers 64 contiguous bytes. Two exchange stages (lane ^ 1, lane ^ 2), one DPP
      // move and three selects per pair of registers.
      const BufferDesc adesc = make_buffer(p.save_in + (size_t)blk * m * d, (size_t)m * d * sizeof(float));
      const int b = i & 3;
      const bool odd = (b & 1) != 0, upper = (b & 2) != 0;
      const int colq = blockIdx.x * kTileCols + (i & ~3);  // first column of the quad
#pragma unroll
      for (int g = 0; g < kTileGroups; ++g) {
        float pc[4][4];  // [piece][element]
#pragma unroll
        for (int pp = 0; pp < 2; ++pp) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float a0 = A[4 * g + r][2 * pp], a1 = A[4 * g + r][2 * pp + 1];
            // one exchange: odd lanes hand over their piece 2pp and get the partner's piece 2pp + 1 (the move itself
            // is unconditional: inside a divergent branch it would read lanes that are switched off)
            const float got = dpp_move<kDppQuadXor1>(odd ? a0 : a1);
            pc[2 * pp][r] = odd ? got : a0;
            pc[2 * pp + 1][r] = odd ? a1 : got;
          }
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float x0 = pc[c][r], x1 = pc[c + 2][r];
            const float got = dpp_move<kDppQuadXor2>(upper ? x0 : x1);  // lanes 2, 3 hand over piece c, get piece c + 2
            pc[c][r] = upper ? got : x0;
            pc[c + 2][r] = upper ? x1 : got;
          }
        }
        const int x = group_x(g) + 16 * q + 4 * b;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const unsigned off = (colq + t < m && x < d) ? ((unsigned)(colq + t) * (unsigned)d + (unsigned)x) * 4u : kOob;
          BufVec<4> v;
          v.e[0] = pc[t][0]; v.e[1] = pc[t][1]; v.e[2] = pc[t][2]; v.e[3] = pc[t][3];
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
#define FASTH_TILE_MIN_COLS 1025  // up to 1024 columns the per-column kernel is faster (three workgroups per compute unit)
#endif
static bool chain_uses_tile(const ChainArgs& a) {
  return a.m >= FASTH_TILE_MIN_COLS && a.d % 4 == 0 && a.d <= kTileMaxD && a.k % kTileRows == 0 &&
         (size_t)a.d * a.m * sizeof(float) < kOob && (size_t)a.n * a.d * sizeof(float) < kOob;  // 32-bit byte offsets
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
    static const std::string name_ = variant_name("chain_tile_kernel", {WW, GG});                           \
    prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, name_.c_str());                                             \
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

}  // namespace fasth
