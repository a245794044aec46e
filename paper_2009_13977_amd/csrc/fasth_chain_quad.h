// Algorithm 1 Step 2 and Algorithm 2 Step 1 for mini-batches of a few hundred columns: chain_quad_kernel, four
// columns per workgroup on the matrix cores. Included by fasth_chain.h (the library has a single translation unit).
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// Between the per-column kernels (one workgroup per column: more columns than compute units run in rounds, and
// every workgroup streams all of V for its one column) and chain_tile_kernel (16 columns per workgroup: fewer than
// 4096 columns leave compute units idle) sits the range 256 < m <= 1024. Here a workgroup of 8 waves takes FOUR
// columns, so a row of V fetched once serves four columns and 1024 columns are one round of 256 workgroups.
//
// v_mfma_f32_4x4x1_16b_f32 computes 16 independent 4 x 4 outer products D_b(v, j) += A_b(v) B_b(j); lane 4 b + i
// supplies A_b(i) and B_b(i) and owns D_b(0..3, i). A_b is always the four columns of the mini-batch (shared by
// groups of blocks through the instruction's broadcast field, so only four lanes per group fetch it), B_b a run of
// four rows of V (first product, C = op(T) B) or four elements x of a row (update): one instruction covers
// 64 rows (or x) times 4 columns for one inner index.
//
// Wave w owns x in [128 w, 128 w + 128) for the whole chain: lane l holds a(128 w + 64 s + l, 0..3), s = 0, 1, in
// accumulators. A step is 32 rows of V (blocks of 64 or 128 rows: the diagonal 32 x 32 blocks of T_i are the steps'
// factors). The wave keeps ITS columns of the step's rows in LDS (32 x 128 floats, fetched one step ahead into
// registers by the wave itself, so these tiles need no barrier), reads them row-wise for B = V a (lane = row and
// half of the x range) and element-wise for a -= V^T C (lane = x). The one barrier of a step is where the 8 partial
// B (32 x 4) meet; every wave then forms C = op(T) B itself (16 instructions), already in operand layout.
// ------------------------------------------------------------------------------------------

constexpr int kQuadWaves = 8, kQuadCols = 4, kQuadRows = 32;
constexpr int kQuadLdv = 1024 + 4;   // row stride of the V tile
constexpr int kQuadLda = 1024 + 4;   // row stride of the transposed activation
constexpr int kQuadLdb = 36;         // row stride of a wave's 4 x 32 scratch

static size_t quad_lds_bytes() {
  return sizeof(float) * ((size_t)kQuadRows * kQuadLdv + (size_t)kQuadCols * kQuadLda +
                          2 * (size_t)kQuadWaves * kQuadRows * kQuadCols + (size_t)kQuadWaves * kQuadCols * kQuadLdb);
}

// A operand of block 0 of each half of the wave (lanes 0..3 and 32..35) used by the 8 blocks of that half.
__device__ __forceinline__ f32x4 mfma4_half(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 3, 0, 0);
}
// A operand of block 0 (lanes 0..3) used by all 16 blocks.
__device__ __forceinline__ f32x4 mfma4_all(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 4, 0, 0);
}

__global__ void __launch_bounds__(64 * kQuadWaves) chain_quad_kernel(ChainArgs p) {
  constexpr int NW = kQuadWaves, K = kQuadRows, LDV = kQuadLdv, LDA = kQuadLda, LDB = kQuadLdb;
  constexpr int XW = 1024 / NW;       // x per wave (256)
  constexpr int XS = XW / 64;         // sets of 64 x per wave in the update (4)
  constexpr int XH = XW / 2;          // x per half of the wave in the first product (128)
  extern __shared__ __align__(16) float smem[];
  float* Vs = smem;                       // [32][LDV]: the step's rows; wave w reads and writes columns XW w .. + XW - 1 only
  float* As = Vs + K * LDV;               // [4][LDA]: the activation, transposed; wave w its own x range only
  float* Bp = As + 4 * LDA;               // [2][NW][32][4]: partial B of every wave, alternating between two buffers
  float* Sc = Bp + 2 * NW * K * 4;        // [NW][4][LDB]: per-wave scratch: B summed, then minus C, both transposed
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int d = p.d, m = p.m, n = p.n;
  const int col0 = blockIdx.x * 4;
  const int xw = XW * wave;                    // this wave's x range
  const int r = lane & 31, h = lane >> 5;      // first product and C: row of the step, half of the inner range
  float* sc = Sc + wave * 4 * LDB;
  const int sub = p.sub, steps = p.nb;         // steps per block; steps of the whole chain (set by the launcher)
  const int ldt = p.kp;                        // row stride of a stored factor
  const float* opT = p.transpose ? p.Tt : p.T;
  auto step_row0 = [&](int s) {                // first row of V of step s
    const int blk = s / sub, part = s % sub;
    const int i = p.transpose ? blk : steps / sub - 1 - blk;
    const int pt = p.transpose ? part : sub - 1 - part;  // within a block the steps go the same way as the blocks
    return i * p.k + pt * K;
  };
  // The wave's columns of a step's 32 rows, RPF rows per fetch: lane l takes row (l / LPR) of the fetch's rows and
  // x = xw + 4 (l % LPR) .. + 3. One per-lane offset serves all fetches (the first row goes into the scalar offset),
  // which keeps the address registers few.
  constexpr int LPR = XW / 4, RPF = 64 / LPR, NF = K / RPF;  // lanes per row, rows per fetch, fetches per step
  const int fx = xw + 4 * (lane % LPR), frow = lane / LPR;
  const unsigned row_off = fx < d ? (unsigned)(frow * d + fx) * 4u : kOob;
  auto rows_of = [&](int s) { return make_buffer(p.V + (size_t)step_row0(s) * d, (size_t)K * d * sizeof(float)); };
  auto fetch_row = [&](BufferDesc vdesc, int j) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(vdesc, row_off, (unsigned)(j * RPF * d) * 4u, 0));
  };
  // this lane's 16 entries of its row of the step's factor: op(T)(r, 16 h .. 16 h + 15)
  auto fetch_t = [&](int s, f32x4 (&tt)[4]) {
    const int row0 = step_row0(s);
    const int blk_row = row0 % p.k, i = row0 / p.k;
    const float* src = opT + (size_t)i * ldt * ldt + (size_t)(blk_row + r) * ldt + blk_row + 16 * h;
#pragma unroll
    for (int q = 0; q < 4; ++q) tt[q] = *reinterpret_cast<const f32x4*>(src + 4 * q);
  };

  // the four columns of the input, with the optional diagonal factor: accumulators and the transposed copy
  f32x4 a[XS];
#pragma unroll
  for (int s2 = 0; s2 < XS; ++s2) {
    const int x = xw + 64 * s2 + lane;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float v = 0.f;
      if (x < d && x < p.in_rows && col0 + c < m) {
        v = p.in[(size_t)x * m + col0 + c];
        if (p.in_scale_mode) v *= diag_factor(p.in_scale_mode, p.in_scale[x]);
      }
      a[s2][c] = v;
      As[c * LDA + x] = v;
    }
  }
  f32x4 stage[NF], tcur[4];
  auto stash = [&](int j) { *reinterpret_cast<f32x4*>(Vs + (j * RPF + frow) * LDV + fx) = stage[j]; };
  {
    const BufferDesc v0desc = rows_of(0);
#pragma unroll
    for (int j = 0; j < NF; ++j) stage[j] = fetch_row(v0desc, j);
  }
  fetch_t(0, tcur);
#pragma unroll
  for (int j = 0; j < NF; ++j) stash(j);
  // (a wave reads only what it wrote itself of Vs and As: LDS operations of one wave complete in order)

  for (int s = 0; s < steps; ++s) {
    const int row0 = step_row0(s);
    const bool more = s + 1 < steps;
    // The next step's rows are fetched, and this block's input saved, between the matrix instructions of the first
    // product: a wave-wide fetch or store costs the compute unit's address unit 16 clocks and holds the issuing
    // wave for longer, while four matrix instructions keep the matrix core busy for 50; issued in one burst at the
    // step's start the same traffic took a microsecond in which no wave computed anything.
    const BufferDesc vnext = rows_of(more ? s + 1 : s);
    const bool saving = p.save_in && s % sub == 0;
    // a buffer over the block's saved columns that exist; elements beyond d are stored nowhere
    const BufferDesc sdesc = make_buffer(p.save_in + ((size_t)(row0 / p.k) * m + col0) * d,
                                         saving ? (size_t)min(4, m - col0) * d * sizeof(float) : 0);
    // ---- B_part(r, c) = sum over this wave's x of V(r, x) a(x, c); lanes 32..63 take the upper half of the range.
    // Chunks of 32 inner indices; the reads of a chunk are issued before the matrix instructions of the chunk
    // before it, so the trip to LDS is hidden behind 32 instructions.
    f32x4 b;
    {
      const float* vrow = Vs + r * LDV + xw + XH * h;
      const float* arow = As + (lane & 3) * LDA + xw + XH * h;
      constexpr int NCH = XH / 32;
      f32x4 vv[2][8], aa[2][8];
      auto read_chunk = [&](int ch, f32x4 (&v8)[8], f32x4 (&a8)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v8[i] = *reinterpret_cast<const f32x4*>(vrow + 32 * ch + 4 * i);
        if ((lane & 31) < 4) {
#pragma unroll
          for (int i = 0; i < 8; ++i) a8[i] = *reinterpret_cast<const f32x4*>(arow + 32 * ch + 4 * i);
        }
      };
      f32x4 acc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      read_chunk(0, vv[0], aa[0]);
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        if (ch + 1 < NCH) read_chunk(ch + 1, vv[(ch + 1) & 1], aa[(ch + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
#pragma unroll
          for (int u = 0; u < 4; ++u) acc[u] = mfma4_half(aa[ch & 1][i][u], vv[ch & 1][i][u], acc[u]);
          __builtin_amdgcn_sched_barrier(0);
          static_assert(NF == 8 * NCH, "one fetch per group of four matrix instructions");
          stage[8 * ch + i] = fetch_row(vnext, 8 * ch + i);
          if (i % 2 == 1) {  // XS * 4 stores per step, one after every second group
            static_assert(XS * 4 == NCH * 4, "one store per odd group");
            const int t = 4 * ch + i / 2, s2 = t / 4, c = t % 4;
            const int x = xw + 64 * s2 + lane;
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(a[s2][c]), sdesc, x < d ? (unsigned)x * 4u : kOob, (unsigned)(c * d) * 4u, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      b = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
      for (int c = 0; c < 4; ++c) b[c] += __shfl_xor(b[c], 32, 64);  // the two halves of the x range
    }
    float* bp = Bp + (s & 1) * NW * K * 4;
    if (lane < 32) *reinterpret_cast<f32x4*>(bp + (wave * K + r) * 4) = b;
    lds_barrier();
    // ---- every wave: B = sum of the partials (fixed order), transposed into its scratch ------------------------
    {
      const int rr = lane >> 1, cc = 2 * (lane & 1);
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float2 v = *reinterpret_cast<const float2*>(bp + (w * K + rr) * 4 + cc);
        s0 += v.x; s1 += v.y;
      }
      sc[cc * LDB + rr] = s0;
      sc[(cc + 1) * LDB + rr] = s1;
    }
    // ---- C(r, c) = sum_l op(T)(r, l) B(l, c): lanes 32..63 take l = 16 .. 31 ----------------------------------
    f32x4 cf;
    {
      f32x4 bb[4];
      if ((lane & 31) < 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q) bb[q] = *reinterpret_cast<const f32x4*>(sc + (lane & 3) * LDB + 16 * h + 4 * q);
      }
      __builtin_amdgcn_sched_barrier(0);
      f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u & 1] = mfma4_half(bb[q][u], tcur[q][u], acc[u & 1]);
      cf = acc[0] + acc[1];
#pragma unroll
      for (int c = 0; c < 4; ++c) cf[c] += __shfl_xor(cf[c], 32, 64);
    }
    if (more) fetch_t(s + 1, tcur);  // the current factor has been used
    if (lane < 32) {
#pragma unroll
      for (int c = 0; c < 4; ++c) sc[c * LDB + r] = -cf[c];  // after this wave's reads of B above (same wave: in order)
      if (p.save_c && wave == 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (col0 + c < m) p.save_c[(size_t)(col0 + c) * n + row0 + r] = cf[c];
      }
    }
    // ---- a(x, c) -= sum_r V(r, x) C(r, c): lane = x, the wave's XS sets of 64 x; chunks of 8 rows, read one
    // chunk ahead; the rows of a chunk that has been used are overwritten with the next step's
    {
      float vv[2][XS][8];
      f32x4 cc[2][2];
      auto read_chunk = [&](int ch, float (&v8)[XS][8], f32x4 (&c2)[2]) {
        if (lane < 4) {
          c2[0] = *reinterpret_cast<const f32x4*>(sc + lane * LDB + 8 * ch);
          c2[1] = *reinterpret_cast<const f32x4*>(sc + lane * LDB + 8 * ch + 4);
        }
#pragma unroll
        for (int rr = 0; rr < 8; ++rr)
#pragma unroll
          for (int s2 = 0; s2 < XS; ++s2) v8[s2][rr] = Vs[(8 * ch + rr) * LDV + xw + 64 * s2 + lane];
      };
      read_chunk(0, vv[0], cc[0]);
#pragma unroll
      for (int ch = 0; ch < 4; ++ch) {
        if (ch + 1 < 4) read_chunk(ch + 1, vv[(ch + 1) & 1], cc[(ch + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int rr = 0; rr < 8; ++rr)
#pragma unroll
          for (int s2 = 0; s2 < XS; ++s2) a[s2] = mfma4_all(cc[ch & 1][rr >> 2][rr & 3], vv[ch & 1][s2][rr], a[s2]);
        __builtin_amdgcn_sched_barrier(0);
        if (more && ch > 0) {  // rows 8 (ch - 1) .. + 7 were read a chunk ago (LDS operations of one wave complete in order)
#pragma unroll
          for (int j = 8 / RPF * (ch - 1); j < 8 / RPF * ch; ++j) stash(j);
        }
      }
      if (more) {
#pragma unroll
        for (int j = 24 / RPF; j < NF; ++j) stash(j);
      }
    }
#pragma unroll
    for (int s2 = 0; s2 < XS; ++s2)
#pragma unroll
      for (int c = 0; c < 4; ++c) As[c * LDA + xw + 64 * s2 + lane] = a[s2][c];
  }
#pragma unroll
  for (int s2 = 0; s2 < XS; ++s2) {
    const int x = xw + 64 * s2 + lane;
    if (x < d) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (col0 + c < m) p.out[(size_t)x * m + col0 + c] = a[s2][c];
    }
  }
}

// Shapes the four-column chain serves, and where it is the faster one. Its time hardly depends on the number of
// columns (one round of up to 256 workgroups: d = n = 1024, k = 32, forward + backward: 283 us at m = 384, 372 us
// at m = 1024), while the per-column kernels run in rounds of 256 to 768 columns: measured against them in the same
// run it wins from 769 columns on (m = 800: 423 -> 331 us at d = 1024, 298 -> 251 us at d = 768, 242 -> 207 us at
// d = 640; m = 1024: 478 -> 372, 330 -> 271, 268 -> 222 us), and at d > 896 from about 600 (m = 640: 324 -> 306 us;
// m = 512: 246 against 295 us, so not there).
#ifndef FASTH_QUAD_MIN_COLS
#define FASTH_QUAD_MIN_COLS 769
#endif
#ifndef FASTH_QUAD_MIN_COLS_LONG
#define FASTH_QUAD_MIN_COLS_LONG 608  // d > 896
#endif
static bool chain_uses_quad(const ChainArgs& a) {
  return (a.m >= FASTH_QUAD_MIN_COLS || (a.d > 896 && a.m >= FASTH_QUAD_MIN_COLS_LONG)) && a.m < FASTH_TILE_MIN_COLS &&
         a.d > 512 && a.d <= 1024 && a.d % 4 == 0 && a.k % kQuadRows == 0 && a.kp == a.k;
}

static int launch_chain_quad(const ChainArgs& args, hipStream_t stream) {
  if (args.d > 1024 || args.d % 4 != 0 || args.k % kQuadRows != 0 || args.kp != args.k || args.n % args.k != 0)
    return FASTH_EINVAL;
  ChainArgs a = args;
  a.sub = args.k / kQuadRows;
  a.nb = args.nb * a.sub;
  const size_t lds = quad_lds_bytes();
  int rc = allow_lds(chain_quad_kernel, lds);
  if (rc != FASTH_OK) return rc;
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, "chain_quad_kernel");
  hipLaunchKernelGGL(chain_quad_kernel, dim3((a.m + kQuadCols - 1) / kQuadCols), dim3(64 * kQuadWaves), lds, stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

}  // namespace fasth
