// Algorithm 1 Step 2 and Algorithm 2 Step 1 on the matrix cores for mini-batches of some hundred columns:
// chain_team_tile_kernel, in which a team of two to four workgroups shares a tile of 16 columns.
// Included by fasth_chain.h (the library has a single translation unit).
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// With a few hundred columns neither form of the chain fills the chip: a workgroup per column runs in rounds on the
// vector units, a workgroup per 16 columns (chain_tile_kernel) leaves most compute units idle. Here the two products
// of a step are matrix products with N = 16 columns on the matrix cores (as in chain_tile_kernel), and a tile of
// 16 columns is shared by NP = ceil(d / 256) workgroups ("parts", 2 to 4) on different compute units: part j keeps
// rows [256 j, 256 j + 256) of the d x 16 tile of A in its accumulator registers for the whole chain and reads only
// those columns of V. A step takes 64 rows (blocks of 32 merged in pairs by the factor kernel, blocks of 64, blocks
// of 128 as two steps with the diagonal blocks of their factor): B = V_rows A is 64 x 16 per step, of which every
// part forms its share over its 256 elements; the parts hand each other their shares through the workspace (each
// to every other, 16-byte words {sum, tag, sum, tag}, tagged and bounded as in chain_team_kernel), add them in the
// order of the parts, and every part forms C = op(T) B (four matrix-core tiles) and updates its rows of A.
// For columns of 1025 to 2048 elements the parts are 512 elements long and a step takes 32 rows (the same registers
// and LDS; blocks of more rows as several steps with the diagonal 32 x 32 blocks of their factor).
//
// Lanes (for parts of 256 elements: NT = 2 accumulator tiles per wave; parts of 512 have NT = 4, 16 NT elements per
// wave likewise). Wave w of the 8 owns 32 elements x_w .. x_w + 31 of the part's 256 as two accumulator tiles r = 0, 1:
// register j of lane (q, i) = (lane / 16, lane % 16) of tile r holds A(x_w + 8 q + 2 j + r, column i). A contraction
// may run over x in any order, so this layout serves as the B operand of the first product (matrix instruction
// (j, r) sums over the four x with the lanes' q) and is the output layout of the second (output row 4 q + j of
// tile r is x_w + 2 (4 q + j) + r) without any shuffle, every fetch of V from LDS is 8 bytes (both tiles' entries),
// and a lane's eight elements of a column are 32 contiguous bytes when a block's input is saved.
// Each wave stages only its own 32 columns of the step's 64 rows in LDS (fetched into registers a step ahead,
// written once its second product has read the old ones), so no barrier guards the rows. Three barriers per step:
// the waves' shares of B meet in LDS (and go out to the other parts), the totals come back into LDS in the layout
// the matrix cores want, and C goes from the waves that form it (each one half of the inner index of some rows) to all.
// ------------------------------------------------------------------------------------------
constexpr int kTtCols = 16;  // columns per team
// NT accumulator tiles (16 NT elements) per wave: 128 NT elements per workgroup, 128 / NT rows per step; row stride of a
// wave's rows in LDS 34 floats (8-byte reads of 16 rows hit 16 bank pairs) or 68 (16-byte reads, aligned)
constexpr size_t kTtLdsFloats = (size_t)8 * 64 * 34 + 8 * 1024 + 1024 + 2 * 1024;
static_assert(8 * 32 * 68 == 8 * 64 * 34, "the rows of a step take the same room in both forms");

// NT = 2: parts of 256 elements, steps of 64 rows; p.sub = 0: the caller's blocks of 32 rows two per step, else steps per
// block (1 or 2). NT = 4: parts of 512 elements, steps of 32 rows, p.sub = 1, 2 or 4 steps per block. LDT = 128 / NT: rows
// of a stored factor, those of a step whatever the caller's block size (the diagonal blocks of a larger block's factor
// are the factors of its row groups, so only those are built). The number of parts is p.parts.
template <int NT, int LDT>
__global__ void __launch_bounds__(512) chain_team_tile_kernel(ChainArgs p) {
  const int NP = p.parts;  // 2 .. 4
  constexpr int K = 128 / NT, RT = K / 16, LD = NT == 2 ? 34 : 68, XW = 16 * NT, SLICE = 8 * XW, F = 4 * NT;
  constexpr int E = RT * 256;  // entries of B per step
  extern __shared__ __align__(16) float smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = lane >> 4, i = lane & 15;
  float* Vs = smem + (size_t)wave * K * LD;  // this wave's 16 NT columns of the step's rows: [K][LD]
  float* Bp = smem + (size_t)8 * K * LD;     // the waves' shares of B: [8][E], element (row 16 rt + 4 q + jj, column i)
                                             // of a wave at ((rt * 64 + lane) * 4 + jj)
  float* Btot = Bp + 8 * 1024;               // B summed over waves and parts, [K][16]
  float* Cs = Btot + 1024;                   // C in two shares (one per half of the inner index), [2][K][16] (second share at 1024)
  const int m = p.m, d = p.d, n = p.n;
  const int tiles = (m + kTtCols - 1) / kTtCols;
  // workgroups b, b + 8, ... (one XCD) are the parts of tile 8 (b / (8 NP)) + b % 8
  const int chain_wgs = 8 * NP * ((tiles + 7) / 8);
  if ((int)blockIdx.x >= chain_wgs) {  // the side product, on compute units the chain leaves idle
    const int row = ((int)blockIdx.x - chain_wgs) * 8 + wave;
    if (row < p.ds_rows) dsigma_row(p.in, p.ds_z1, p.in_scale, p.ds_out, row, m, p.in_scale_mode);
    return;
  }
  const int part = (int)(blockIdx.x >> 3) % NP;
  const int tile = (int)(blockIdx.x >> 3) / NP * 8 + (int)(blockIdx.x & 7);
  if (tile >= tiles) return;
  const int col = tile * kTtCols + i;
  const bool col_ok = col < m;
  const int x_w = part * SLICE + XW * wave;  // this wave's first element

  // the input tile: rows beyond those that exist and columns beyond m read as zero
  f32x4 A[NT];
  {
    const BufferDesc xdesc = make_buffer(p.in, (size_t)p.in_rows * m * sizeof(float));
#pragma unroll
    for (int r = 0; r < NT; ++r) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int x = x_w + F * q + NT * j + r;
        const unsigned off = col_ok && x < p.in_rows ? ((unsigned)x * (unsigned)m + (unsigned)col) * 4u : kOob;
        A[r][j] = buffer_load<1>(xdesc, off, 0).e[0];
      }
    }
    if (p.in_scale_mode) {
      // all fetches first, then the mode as a compile-time constant: rows that do not exist hold zero in A already;
      // their sigma is replaced by 1 so that the factor stays finite
      const BufferDesc sdesc = make_buffer(p.in_scale, (size_t)p.in_rows * sizeof(float));
      f32x4 sg[NT];
#pragma unroll
      for (int r = 0; r < NT; ++r) {
#pragma unroll
        for (int j = 0; j < 4; ++j) sg[r][j] = buffer_load<1>(sdesc, (unsigned)(x_w + F * q + NT * j + r) * 4u, 0).e[0];
      }
      auto scale_rows = [&](auto mode) {
#pragma unroll
        for (int r = 0; r < NT; ++r) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float sv = x_w + F * q + NT * j + r < p.in_rows ? sg[r][j] : 1.f;
            A[r][j] *= diag_factor(decltype(mode)::value, sv);
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
  }

  const BufferDesc hdesc = make_buffer(reinterpret_cast<const float*>(p.xch + (size_t)tile * team_tile_words(NP)),
                                       team_tile_words(NP) * 4u);
  const unsigned tag0 = __builtin_amdgcn_raw_buffer_load_b32(hdesc, 0u, 0, 16);
  bool gave_up = false, same_xcd = false;
  const unsigned my_xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;
  const unsigned hs_tag = tag0 + 1u;
  if (tid == 0) {
    const u32x2 w = {my_xcc, hs_tag};
    __builtin_amdgcn_raw_buffer_store_b64(w, hdesc, 32u + (unsigned)part * 8u, 0, 16);
  }

  // staging of a step's rows: lane l fetches 16 bytes at x = x_w + 4 (l % F) of rows (64 / F) u + l / F, u < 8
  const BufferDesc vdesc = make_buffer(p.V, (size_t)n * d * sizeof(float));
  const int srow = lane / F, sx = x_w + 4 * (lane % F);
  const unsigned stage_off = sx < d ? ((unsigned)srow * (unsigned)d + (unsigned)sx) * 4u : kOob;
  BufVec<4> stage[8];
  auto fetch_rows = [&](int row0) {
#pragma unroll
    for (int u = 0; u < 8; ++u) stage[u] = buffer_load<4>(vdesc, stage_off, (unsigned)(row0 + (64 / F) * u) * (unsigned)d * 4u);
  };
  auto stash_rows = [&]() {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      float* dst = Vs + ((64 / F) * u + srow) * LD + 4 * (lane % F);
      if constexpr (NT == 4) {
        *reinterpret_cast<float4*>(dst) = make_float4(stage[u].e[0], stage[u].e[1], stage[u].e[2], stage[u].e[3]);
      } else {
        *reinterpret_cast<float2*>(dst) = make_float2(stage[u].e[0], stage[u].e[1]);
        *reinterpret_cast<float2*>(dst + 2) = make_float2(stage[u].e[2], stage[u].e[3]);
      }
    }
  };
  // op(T) of step st as the A operand of C = op(T) B. Wave w < 2 RT forms rows 16 (w % RT) .. + 15 of C from half w / RT
  // of the inner index, K / 8 matrix instructions; instruction kk sums over the inner indices
  // (K / 2) (w / RT) + (K / 8) q + kk (the sum may run in any order), so lane (q, i) needs K / 8 consecutive entries of
  // its row. (The other waves fetch what wave w % (2 RT) does and do not use it: no branch.)
  constexpr int TN = K / 8;
  const int crt = wave % RT, chalf = (wave / RT) & 1;
  const int sub = p.sub;  // steps per block; 0: two blocks per step
  auto fetch_t = [&](int st, float (&t)[TN]) {
    const float* opT = p.transpose ? p.Tt : p.T;
    const float* Ts = opT + (size_t)st * LDT * LDT;  // a stored factor has the rows of a step
    const float4* src = reinterpret_cast<const float4*>(Ts + (16 * crt + i) * LDT + (K / 2) * chalf + TN * q);
#pragma unroll
    for (int g = 0; g < TN / 4; ++g) {
      const float4 v = src[g];
      t[4 * g] = v.x; t[4 * g + 1] = v.y; t[4 * g + 2] = v.z; t[4 * g + 3] = v.w;
    }
  };
  // A lane's 4 NT elements of column i are contiguous in the saved input
  auto save_input = [&](int block) {
    if (!p.save_in) return;
    const BufferDesc adesc = make_buffer(p.save_in + (size_t)block * m * d, (size_t)m * d * sizeof(float));
    const int x = x_w + F * q;
#pragma unroll
    for (int h = 0; h < NT; ++h) {
      BufVec<4> v;
      if constexpr (NT == 4) {
        v.e[0] = A[0][h]; v.e[1] = A[1][h]; v.e[2] = A[2][h]; v.e[3] = A[3][h];
      } else {
        v.e[0] = A[0][2 * h]; v.e[1] = A[1][2 * h]; v.e[2] = A[0][2 * h + 1]; v.e[3] = A[1][2 * h + 1];
      }
      const unsigned off = col_ok && x + 4 * h < d ? ((unsigned)col * (unsigned)d + (unsigned)(x + 4 * h)) * 4u : kOob;
      buffer_store<4>(adesc, off, 0, v);
    }
  };

  const int ns = n / K;
  auto step_of = [&](int s) { return p.transpose ? s : ns - 1 - s; };
  float tcur[TN], tnxt[TN];
  fetch_rows(step_of(0) * K);
  fetch_t(step_of(0), tcur);
  stash_rows();
  {
    unsigned peer_xcc = my_xcc;
    const unsigned hs_from = 32u + (unsigned)(lane < NP ? lane : part) * 8u;
    int polls = 0;
    for (;;) {
      const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(hdesc, hs_from, 0, 16);
      peer_xcc = w.x;
      if (__all(w.y == hs_tag)) break;
      if (polls++ >= p.wait_limit) { gave_up = true; break; }
      asm volatile("" ::: "memory");
    }
    same_xcd = !gave_up && __all(peer_xcc == my_xcc);
  }
  for (int s = 0; s < ns; ++s) {
    const int st = step_of(s), stn = step_of(s + 1 < ns ? s + 1 : s);
    fetch_rows(stn * K);
    fetch_t(stn, tnxt);
    // the input of the caller's block that this step starts with
    if (sub == 0) save_input(2 * st + (p.transpose ? 0 : 1));
    else if (st % sub == (p.transpose ? 0 : sub - 1)) save_input(st / sub);
    // this wave's share of B = V_rows A: rows 16 rt .. 16 rt + 15 in acc[rt]
    f32x4 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float* vp = Vs + (16 * rt + i) * LD + F * q + NT * j;
        if constexpr (NT == 4) {
          const float4 v = *reinterpret_cast<const float4*>(vp);
          acc[rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.x, A[0][j], acc[rt], 0, 0, 0);
          acc[rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.y, A[1][j], acc[rt], 0, 0, 0);
          acc[rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.z, A[2][j], acc[rt], 0, 0, 0);
          acc[rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.w, A[3][j], acc[rt], 0, 0, 0);
        } else {
          const float2 v = *reinterpret_cast<const float2*>(vp);
          acc[rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.x, A[0][j], acc[rt], 0, 0, 0);
          acc[rt] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.y, A[1][j], acc[rt], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) *reinterpret_cast<f32x4*>(Bp + ((size_t)(wave * RT + rt) * 64 + lane) * 4) = acc[rt];
    lds_barrier();
    if (2 * tid < E) {
      // thread t < E / 2 adds entries 2 t, 2 t + 1 of the eight waves' shares, sends the sums to the other parts, receives
      // theirs (whole waves: E / 2 is a multiple of 64)
      float2 own = *reinterpret_cast<const float2*>(Bp + 2 * tid);
#pragma unroll
      for (int w = 1; w < 8; ++w) {
        const float2 o = *reinterpret_cast<const float2*>(Bp + w * E + 2 * tid);
        own.x += o.x; own.y += o.y;
      }
      const unsigned tag = tag0 + 1u + (unsigned)s, par = (unsigned)s & 1u;
      const u32x4 out = {__builtin_bit_cast(unsigned, own.x), tag, __builtin_bit_cast(unsigned, own.y), tag};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j < NP && j != part) {
          const unsigned to = (unsigned)kTeamHeadBytes + ((((unsigned)j * 2u + par) * NP + (unsigned)part) * 512u + (unsigned)tid) * 16u;
          if (same_xcd) __builtin_amdgcn_raw_buffer_store_b128(out, hdesc, to, 0, 0);
          else __builtin_amdgcn_raw_buffer_store_b128(out, hdesc, to, 0, 16);
        }
      }
      float g0[4], g1[4];  // part j's sums (zero once a wait has given up)
#pragma unroll
      for (int j = 0; j < 4; ++j) { g0[j] = 0.f; g1[j] = 0.f; }
      if (!gave_up) {
        int polls = 0;
        for (;;) {
          bool all_in = true;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (j < NP && j != part) {
              const unsigned from = (unsigned)kTeamHeadBytes + ((((unsigned)part * 2u + par) * NP + (unsigned)j) * 512u + (unsigned)tid) * 16u;
              // (the word is declared inside the loop and its entries copied out one by one on purpose)
              const u32x4 w = same_xcd ? __builtin_amdgcn_raw_buffer_load_b128(hdesc, from, 0, 2)
                                       : __builtin_amdgcn_raw_buffer_load_b128(hdesc, from, 0, 16);
              const unsigned t0 = w.y, t1 = w.w;
              g0[j] = __builtin_bit_cast(float, (unsigned)w.x);
              g1[j] = __builtin_bit_cast(float, (unsigned)w.z);
              all_in = all_in && t0 == tag && t1 == tag;
            }
          }
          if (__all(all_in)) break;
          if (polls++ >= p.wait_limit) { gave_up = true; break; }
          asm volatile("" ::: "memory");
        }
      }
      // the parts' sums in the order of the parts: every part gets the same bits
      float2 total = make_float2(0.f, 0.f);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j < NP) {
          total.x += j == part ? own.x : g0[j];
          total.y += j == part ? own.y : g1[j];
        }
      }
      // entries 2 t, 2 t + 1 are rows 16 rt + 4 q' + jj, jj = 2 (t % 2) + {0, 1}, of column i' (rt = t / 128, 16 q' + i' = t / 2 % 64)
      const int row = 16 * (tid >> 7) + 4 * ((tid >> 5) & 3) + 2 * (tid & 1), c = (tid >> 1) & 15;
      Btot[row * 16 + c] = total.x;
      Btot[(row + 1) * 16 + c] = total.y;
    }
    lds_barrier();
    if (wave < 2 * RT) {
      // this wave's share of C: rows 16 (w % RT) .., half w / RT of the inner index; the two shares of a row meet when they are read
      f32x4 C0 = {0.f, 0.f, 0.f, 0.f}, C1 = {0.f, 0.f, 0.f, 0.f};
      const float* bsrc = Btot + ((K / 2) * chalf + TN * q) * 16 + i;
#pragma unroll
      for (int kk = 0; kk < TN; kk += 2) {
        C0 = __builtin_amdgcn_mfma_f32_16x16x4f32(tcur[kk], bsrc[kk * 16], C0, 0, 0, 0);
        C1 = __builtin_amdgcn_mfma_f32_16x16x4f32(tcur[kk + 1], bsrc[(kk + 1) * 16], C1, 0, 0, 0);
      }
      const f32x4 C = C0 + C1;
      float* cdst = Cs + chalf * 1024 + (16 * crt + 4 * q) * 16 + i;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) cdst[jj * 16] = C[jj];
    }
    lds_barrier();
    if (p.save_c && part == 0 && wave < RT) {
      // wave w saves rows 16 w .. 16 w + 15 of C: lane (q, i) rows 4 q .. 4 q + 3 of column i
      float c4[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) c4[jj] = Cs[(16 * wave + 4 * q + jj) * 16 + i] + Cs[1024 + (16 * wave + 4 * q + jj) * 16 + i];
      if (col_ok) *reinterpret_cast<float4*>(p.save_c + (size_t)col * n + (size_t)st * K + 16 * wave + 4 * q) = make_float4(c4[0], c4[1], c4[2], c4[3]);
    }
    // A -= V_rows^T C, the half of the step that is applied first before the other (the later rows first in the plain order)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int half = p.transpose ? hh : 1 - hh;
#pragma unroll
      for (int rr = 0; rr < RT / 2; ++rr) {
        const int rt = (RT / 2) * half + rr;
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) {
          const int row = 16 * rt + 4 * q + s2;
          const float cneg = -(Cs[row * 16 + i] + Cs[1024 + row * 16 + i]);
          const float* vp = Vs + row * LD + NT * i;
          if constexpr (NT == 4) {
            const float4 v = *reinterpret_cast<const float4*>(vp);
            A[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.x, cneg, A[0], 0, 0, 0);
            A[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.y, cneg, A[1], 0, 0, 0);
            A[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.z, cneg, A[2], 0, 0, 0);
            A[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.w, cneg, A[3], 0, 0, 0);
          } else {
            const float2 v = *reinterpret_cast<const float2*>(vp);
            A[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.x, cneg, A[0], 0, 0, 0);
            A[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(v.y, cneg, A[1], 0, 0, 0);
          }
        }
      }
      // two blocks of 32 in a step of 64: the state between the halves is the input of the pair's other block
      if (sub == 0 && hh == 0) save_input(2 * st + (p.transpose ? 1 : 0));
    }
    stash_rows();
#pragma unroll
    for (int kk = 0; kk < TN; ++kk) tcur[kk] = tnxt[kk];
  }
  // the next launch on this workspace counts on from here
  if (part == 0 && tid == 0) __builtin_amdgcn_raw_buffer_store_b32(tag0 + (unsigned)ns, hdesc, 0u, 0, 16);
  if (gave_up && lane == 0) __hip_atomic_store(&g_wait_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  {
    const BufferDesc odesc = make_buffer(p.out, (size_t)d * m * sizeof(float));
#pragma unroll
    for (int r = 0; r < NT; ++r) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int x = x_w + F * q + NT * j + r;
        BufVec<1> v;
        v.e[0] = A[r][j];
        buffer_store<1>(odesc, col_ok && x < d ? ((unsigned)x * (unsigned)m + (unsigned)col) * 4u : kOob, 0, v);
      }
    }
  }
}

static bool chain_uses_team_tile(const ChainArgs& a) { return a.xch != nullptr && team_tile_parts(a.d, a.n, a.m, a.k) > 0; }

static int launch_chain_team_tile(const ChainArgs& args, hipStream_t stream) {
  ChainArgs a = args;
  a.parts = team_tile_parts(a.d, a.n, a.m, a.k);
  if (a.parts == 0 || !a.xch) return FASTH_EINVAL;
  const bool longer = a.d > 1024;  // parts of 512 elements, steps of 32 rows
  // steps per block (0: two of the caller's blocks of 32 per step of 64 rows)
  a.sub = longer ? a.k / 32 : a.k == 32 ? 0 : a.k / 64;
  const size_t lds = kTtLdsFloats * sizeof(float);
  const int side = a.ds_out ? (a.ds_rows + 7) / 8 : 0;
  const int tiles = (a.m + kTtCols - 1) / kTtCols;
  const dim3 grid(8 * a.parts * ((tiles + 7) / 8) + side), block(512);
#define FASTH_LAUNCH_TT(NT_, LDT_)                                                                                   \
  do {                                                                                                               \
    int rc_ = allow_lds(chain_team_tile_kernel<NT_, LDT_>, lds);                                                     \
    if (rc_ != FASTH_OK) return rc_;                                                                                 \
    static const std::string names_[3] = {variant_name("chain_team_tile_kernel", {NT_, LDT_}) + " (2 parts)",         \
                                          variant_name("chain_team_tile_kernel", {NT_, LDT_}) + " (3 parts)",         \
                                          variant_name("chain_team_tile_kernel", {NT_, LDT_}) + " (4 parts)"};        \
    prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, names_[a.parts - 2].c_str());                                        \
    hipLaunchKernelGGL((chain_team_tile_kernel<NT_, LDT_>), grid, block, lds, stream, a);                            \
  } while (0)
  if (!longer) FASTH_LAUNCH_TT(2, 64);
  else FASTH_LAUNCH_TT(4, 32);
#undef FASTH_LAUNCH_TT
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

}  // namespace fasth
