// Algorithm 1 Step 2 and Algorithm 2 Step 1 for d <= 1024 (a multiple of 4) and blocks of 32, 64 or 128 rows:
// chain_pair_kernel, the per-column chain in which pairs of lanes share a chunk of the column.
// Included by fasth_chain.h.
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// A fetch keeps the wave that issues it from its arithmetic for ~35 clocks, and with one wave per SIMD (the 4-wave
// kernel) nothing else can use the SIMD meanwhile. Eight waves, two per SIMD, can fill each other's stalls; but a
// wave-wide fetch costs the compute unit's address unit the same 16 clocks whether its lanes take 16 or 8 bytes, so
// the eight waves together must not issue more fetches than the four did. Here two lanes share one 16-byte chunk of
// the column (x = 4J .. 4J + 3, both hold the same four elements of `a`) and split the ROWS of a step between them:
// the lane of parity h holds rows 2jj + h of the 32-row step, 16 fetches of 16 bytes per lane and step instead of 32.
//   B = V a:      each lane forms the partial inner products of its 16 rows; they are summed over the 32 lanes of
//                 equal parity (register butterfly that skips the parity bit) and over the waves through LDS.
//   a -= V^T C:   the lane of parity 0 starts from a, the other from 0, each subtracts its 16 rows' terms, and
//                 the two exchange their sums with one DPP move per element: x + y = y + x exactly, so both lanes
//                 keep bit-identical copies of a.
// The parity is lane bit 3 and the partner of lane i is lane i ^ 15 of its row of 16 (DPP row_mirror): lanes 0..7 of a
// row take chunks c .. c + 7 of one row of V, lanes 8..15 the same chunks of the next row in reverse order, so 8
// adjacent lanes fetch 128 contiguous bytes, which costs the address unit no more than 1 KiB contiguous per wave
// (lane pairs (2j, 2j + 1) on alternate rows cost twice as much). The butterfly's remaining stages use lane bits
// 5, 4 (permlane swaps) and 2, 1, 0 (DPP half-mirror and quad permutes, none of which changes bit 3).
struct PairLanes {
  static constexpr int M0 = 4, M1 = 2, M2 = 1;  // lane bits below 8 for the last two halving stages and the last sum
  __device__ static __forceinline__ int parity(int lane) { return (lane >> 3) & 1; }
  // chunk of the wave's 32 that the lane works on
  __device__ static __forceinline__ int chunk(int lane) { return 8 * (lane >> 4) + ((lane & 8) ? 7 - (lane & 7) : (lane & 7)); }
  __device__ static __forceinline__ float partner(float x) { return dpp_move<kDppRowMirror>(x); }
};

template <int LPT>
struct PairRegs {
  Chunk<4> v[16];  // this lane's 16 rows of the step, its pair's chunk
  float t[LPT];    // this thread's entries of its row of op(T) of the step
};

// SUB: steps of 32 rows per block (k = 32 SUB; the diagonal 32 x 32 blocks of T_i are the steps' factors).
// PAD: k is not a multiple of 32 and SUB = ceil(k / 32): the last step of a block has fewer than 32 rows; its missing
// rows repeat the last valid one and their inner products and coefficients are forced to zero.
// UNAL (with PAD, and SUB = 0: the steps per block come from p.sub): d is not a multiple of 4, so rows are not
// 16-byte aligned and a row's last chunk hangs over its end. Rows are then fetched through a buffer that spans the
// step's block (4-byte alignment is enough for it, what lies beyond the block reads as zero); the overhanging
// elements of `a` see the next row's values, so they are put back to zero after every update and never stored.
// Three register copies of a step's rows (64 registers each): while step s is applied, the rows of step s + 2 are
// fetched, so every fetch has more than a whole step to arrive and may be issued wherever it costs least.
// Of a lane's 16 fetches per step, P1 are issued during the first product, RL during the reduction, XA after the
// first barrier and XC after the second (while the LDS reads issued there are on their way), the rest during the update.
// NW: waves per workgroup, 128 elements of the column each (8 for d <= 1024, 4 for d <= 512, 2 for d <= 256).
//
// SPLIT: the column is longer than one workgroup's 128 NW elements and TWO workgroups share it, each holding one
// half of the column and of every row of V (half 0: x < 128 NW, half 1: the rest), so that a step keeps its 32 rows
// and each compute unit fetches and multiplies half of them. The only thing the halves owe each other is a step's
// 32 partial inner products: after the sum over its own waves each workgroup hands them to the other through the
// workspace and adds what it receives (x + y = y + x exactly, so both form the same coefficients bit for bit and
// nothing else is exchanged). A hand-off is 16 words of 16 bytes {b[2 t], tag, b[2 t + 1], tag}: each value and its
// "ready" travel in the same 8 bytes, a word is valid once both tags equal the step's, and two sets of words alternate between
// steps (a workgroup cannot be more than one step ahead of its partner, which it waits for in every step). Tags
// count on from launch to launch through a word per column that the factor kernels zero together with the
// hand-off words, so no stale word ever carries a valid tag, also when a captured launch is replayed. Stores and
// loads of the hand-off are agent-scope (correct wherever the two workgroups run); the launch puts partners on one
// XCD (workgroups b and b + 8), where the trip is shortest. Every wait is bounded: after p.wait_limit polls a wave
// gives up for the rest of the launch, raises the library's status word and runs on with what it has, so the
// kernel always ends; fasth_wait_status() tells the host.
template <int NW, int SUB, int P1, int RL, int XA, int XC, bool PAD = false, bool UNAL = false, bool SPLIT = false>
__global__ void __launch_bounds__(64 * NW) chain_pair_kernel(ChainArgs p) {
  static_assert(!UNAL || (PAD && SUB == 0), "the unaligned form is the general one");
  static_assert(!SPLIT || (NW == 8 && !PAD && !UNAL), "two halves of 1024 elements, whole steps, aligned rows");
  static_assert(SUB > 0 || PAD, "steps per block");
  typedef PairLanes Lanes;
  constexpr int K = 32, KH = 16, G = 2 * NW, LPT = K / G;  // G threads share a row of op(T), LPT entries each
  typedef PairRegs<LPT> Regs;
  static_assert(NW == 2 || NW == 4 || NW == 8, "waves");
  constexpr int PR2 = KH - RL - P1 - XA - XC;
  constexpr int S1 = KH / P1, S2 = KH / PR2;
  constexpr int RS = RL > 4 ? 2 : 4;  // one fetch every RS exchanges of the reduction
  constexpr int XA0 = P1 + RL, XC0 = XA0 + XA, U0 = XC0 + XC;
  static_assert(P1 >= 1 && PR2 >= 1 && RL >= 0 && RL <= 8 && XA >= 0 && XC >= 0, "prefetch split");
  __shared__ __align__(16) float Bpart[NW][K];
  __shared__ __align__(16) float Cv[2][KH];  // [parity][jj] = coefficient of row 2 jj + parity
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = p.m, d = p.d;
  // SPLIT: workgroups b and b + 8 (same XCD) are the halves of column 8 (b / 16) + b % 8
  const int half = SPLIT ? (int)(blockIdx.x >> 3) & 1 : 0;
  const int col = SPLIT ? (int)(blockIdx.x >> 4) * 8 + (int)(blockIdx.x & 7) : (int)blockIdx.x;
  if (col >= m) {  // workgroups beyond the columns: the side product, on compute units the chain leaves idle
    if constexpr (!SPLIT) {
      const int row = (col - m) * NW + wave;
      if (row < p.ds_rows) dsigma_row(p.in, p.ds_z1, p.in_scale, p.ds_out, row, m, p.in_scale_mode);
    }
    return;
  }
  const int h = Lanes::parity(lane);
  const unsigned x0w = (unsigned)half * (128u * NW) + 4u * (unsigned)(wave * 32 + Lanes::chunk(lane));
  const bool ok = x0w < (unsigned)d;
  const unsigned x0 = ok ? x0w : 0u;  // lanes beyond d fetch chunk 0 (valid memory) and keep their elements at zero
  const unsigned lane_off = (unsigned)h * (unsigned)d + x0;
  Chunk<4> a = load_column_chunk<4>(p, col, x0, ok);
  const int trow = tid / G, tg = tid % G;
  const int nb = p.nb;
  // SPLIT: per column [2 (receiving half)][2 (step parity)][16] words of 16 bytes, then the tag counter
  BufferDesc xdesc;
  unsigned tag0 = 0, steps_done = 0;
  bool gave_up = false;
  bool same_xcd = false;
  if constexpr (SPLIT) {
    xdesc = make_buffer(reinterpret_cast<const float*>(p.xch + (size_t)col * kSplitPairWords), kSplitPairWords * 4u);
    tag0 = __builtin_amdgcn_raw_buffer_load_b32(xdesc, 1024u, 0, 16);
    // Do the two halves run on one XCD, i.e. behind one L2? Each tells the other the id of its own (agent-scope,
    // tagged like a hand-off) before the chain starts. If they do, the hand-offs use ordinary stores, which that
    // L2 holds, and loads that skip only the compute unit's own cache: a shorter trip than through memory.
    const unsigned my_xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;  // XCC_ID
    const unsigned hs_tag = tag0 + 1u;
    if (tid == 0) {
      const u32x2 w = {my_xcc, hs_tag};
      __builtin_amdgcn_raw_buffer_store_b64(w, xdesc, 1024u + 32u + (unsigned)(1 - half) * 8u, 0, 16);
    }
    unsigned peer_xcc = ~0u;
    int polls = 0;
    for (;;) {
      const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(xdesc, 1024u + 32u + (unsigned)half * 8u, 0, 16);
      peer_xcc = w.x;
      if (__all(w.y == hs_tag)) break;
      if (polls++ >= p.wait_limit) { gave_up = true; break; }
      asm volatile("" ::: "memory");
    }
    same_xcd = !gave_up && peer_xcc == my_xcc;
  }
  const int sel = ((lane & 32) ? 8 : 0) + ((lane & 16) ? 4 : 0) + ((lane & Lanes::M0) ? 2 : 0) + ((lane & Lanes::M1) ? 1 : 0);
  const bool writer = (lane & Lanes::M2) == 0;
  auto block_of = [&](int s) { return p.transpose ? s : nb - 1 - s; };  // step index of the s-th step applied
  const int sub = SUB > 0 ? SUB : p.sub;
  auto step_block = [&](int i) { return SUB == 1 ? i : i / sub; };
  auto step_part = [&](int i) { return SUB == 1 ? 0 : i % sub; };
  bool keep[4];  // elements of this lane's chunk that exist
#pragma unroll
  for (int r = 0; r < 4; ++r) keep[r] = ok && (!UNAL || x0 + r < (unsigned)d);
  auto rows_valid = [&](int i) { return PAD ? min(K, p.k - step_part(i) * K) : K; };
  auto load_row = [&](int i, int jj, Chunk<4>& dst) {
    if constexpr (PAD) {
      // rows 2jj and 2jj + 1 of the step, clamped to its last valid row (scalar arithmetic but for one select)
      const int kv = rows_valid(i);
      const int row0 = step_block(i) * p.k + step_part(i) * K + min(2 * jj, kv - 1);
      const unsigned off = 2 * jj + 1 < kv ? lane_off : x0;
      if constexpr (UNAL) {
        // the buffer spans the step's block of k rows (at most 512 KiB), so V itself may be of any size
        const BufferDesc vdesc = make_buffer(p.V + (size_t)step_block(i) * p.k * d, (size_t)p.k * d * sizeof(float));
        const unsigned row = (unsigned)(step_part(i) * K + min(2 * jj, kv - 1));
        const BufVec<4> v = buffer_load<4>(vdesc, off * 4u, row * (unsigned)d * 4u);
#pragma unroll
        for (int r = 0; r < 4; ++r) dst.e[r] = v.e[r];
      } else {
        dst = load_chunk<4>(p.V + (size_t)row0 * (size_t)d + off);
      }
    } else {
      dst = load_chunk<4>(p.V + ((size_t)i * K + 2 * jj) * (size_t)d + lane_off);
    }
  };
  auto load_t = [&](int i, Regs& r) {
    const int LDT = PAD ? p.kp : K * SUB;  // row stride of the stored factor
    const float* Ti = (p.transpose ? p.Tt : p.T) + (size_t)step_block(i) * LDT * LDT + (size_t)step_part(i) * (K * LDT + K);
    const float* src = Ti + trow * LDT + LPT * tg;
    if constexpr (LPT == 2) {
      const float2 t2 = *reinterpret_cast<const float2*>(src);
      r.t[0] = t2.x; r.t[1] = t2.y;
    } else {
#pragma unroll
      for (int e4 = 0; e4 < LPT / 4; ++e4) {
        const float4 t4 = reinterpret_cast<const float4*>(src)[e4];
        r.t[4 * e4] = t4.x; r.t[4 * e4 + 1] = t4.y; r.t[4 * e4 + 2] = t4.z; r.t[4 * e4 + 3] = t4.w;
      }
    }
  };

  // Applies step i held in `cur` while fetching step ifetch (two steps on) into `dst`.
  auto apply_step = [&](int i, Regs& cur, int ifetch, Regs& dst) {
    if (p.save_in && ok && h == 0 && (SUB == 1 || step_part(i) == (p.transpose ? 0 : sub - 1))) {
      float* dst_in = p.save_in + ((size_t)step_block(i) * m + col) * d + x0;
      if constexpr (UNAL) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (keep[r]) dst_in[r] = a.e[r];
      } else {
        store_chunk<4>(dst_in, a);
      }
    }
    const int kv = rows_valid(i);
    float pj[KH];
#pragma unroll
    for (int jj = 0; jj < KH; ++jj) {
      if (jj % S1 == 0 && jj / S1 < P1) {
        load_row(ifetch, jj / S1, dst.v[jj / S1]);
        __builtin_amdgcn_sched_barrier(0);
      }
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) acc = fmaf(cur.v[jj].e[r], a.e[r], acc);
      pj[jj] = (PAD && 2 * jj + h >= kv) ? 0.f : acc;
    }
    load_t(ifetch, dst);
    auto prefetch = [&](int t) {
      if (t % RS == 0 && t / RS < RL) {
        __builtin_amdgcn_sched_barrier(0);
        load_row(ifetch, P1 + t / RS, dst.v[P1 + t / RS]);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // sum over the 32 lanes of this parity: 16 values, five lane bits
    reduce_stage<KH, 16, 32, 0>(pj, lane, prefetch);
    reduce_stage<KH, 8, 16, 8>(pj, lane, prefetch);
    reduce_stage<KH, 4, Lanes::M0, 12>(pj, lane, prefetch);
    reduce_stage<KH, 2, Lanes::M1, 14>(pj, lane, prefetch);
    reduce_stage<KH, 1, Lanes::M2, 15>(pj, lane, prefetch);
    if (writer) Bpart[wave][2 * sel + h] = pj[0];
    lds_barrier();
    {
      float bw[NW][LPT];
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        if constexpr (LPT == 2) {
          const float2 t2 = *reinterpret_cast<const float2*>(&Bpart[w][LPT * tg]);
          bw[w][0] = t2.x; bw[w][1] = t2.y;
        } else {
#pragma unroll
          for (int e4 = 0; e4 < LPT / 4; ++e4) {
            const float4 t4 = *reinterpret_cast<const float4*>(&Bpart[w][LPT * tg + 4 * e4]);
            bw[w][4 * e4] = t4.x; bw[w][4 * e4 + 1] = t4.y; bw[w][4 * e4 + 2] = t4.z; bw[w][4 * e4 + 3] = t4.w;
          }
        }
      }
      auto fetch_xa = [&]() {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < XA; ++e) load_row(ifetch, XA0 + e, dst.v[XA0 + e]);
        __builtin_amdgcn_sched_barrier(0);
      };
      // fetches while the partial sums are on their way from LDS (SPLIT: behind the hand-off, whose polls would
      // otherwise queue up behind them: loads return in the order they were issued)
      if constexpr (XA > 0 && !SPLIT) fetch_xa();
      float bs[LPT];
#pragma unroll
      for (int e = 0; e < LPT; ++e) {
        float b = bw[0][e];
#pragma unroll
        for (int w = 1; w < NW; ++w) b += bw[w][e];
        bs[e] = b;
      }
      if constexpr (SPLIT) {
        static_assert(LPT == 2, "a hand-off word holds two values");
        const unsigned tag = tag0 + 1u + steps_done, par = (steps_done & 1u) * 256u;
        ++steps_done;
        if (trow == 0) {  // the first 16 threads hold the 32 sums of this half
          const u32x4 w = {__builtin_bit_cast(unsigned, bs[0]), tag, __builtin_bit_cast(unsigned, bs[1]), tag};
          const unsigned to = (unsigned)(1 - half) * 512u + par + (unsigned)tg * 16u;
          if (same_xcd) __builtin_amdgcn_raw_buffer_store_b128(w, xdesc, to, 0, 0);
          else __builtin_amdgcn_raw_buffer_store_b128(w, xdesc, to, 0, 16);
        }
        unsigned r0 = 0u, r1 = 0u;  // the partner's two sums (zero once a wait has given up)
        if (!gave_up) {
          int polls = 0;
          for (;;) {
            const unsigned from = (unsigned)half * 512u + par + (unsigned)tg * 16u;
            const u32x4 w = same_xcd ? __builtin_amdgcn_raw_buffer_load_b128(xdesc, from, 0, 2)
                                     : __builtin_amdgcn_raw_buffer_load_b128(xdesc, from, 0, 16);
            r0 = w.x; r1 = w.z;
            if (__all(w.y == tag && w.w == tag)) break;
            if (polls++ >= p.wait_limit) { gave_up = true; break; }
            asm volatile("" ::: "memory");
          }
        }
        bs[0] += __builtin_bit_cast(float, r0);
        bs[1] += __builtin_bit_cast(float, r1);
        if constexpr (XA > 0) fetch_xa();
      }
      float c = 0.f;
#pragma unroll
      for (int e = 0; e < LPT; ++e) c = fmaf(cur.t[e], bs[e], c);
      c = group_sum<G>(c);
      if (PAD && trow >= kv) c = 0.f;
      if (tg == 0) {
        Cv[trow & 1][trow >> 1] = c;
        if constexpr (PAD) {
          if (p.save_c && trow < kv) p.save_c[(size_t)col * p.n + (size_t)step_block(i) * p.k + step_part(i) * K + trow] = c;
        } else {
          if (p.save_c && half == 0) p.save_c[(size_t)col * p.n + (size_t)i * K + trow] = c;
        }
      }
    }
    lds_barrier();
    float cc[2][8];
    auto read_cc = [&](int grp, float (&out)[8]) {
#pragma unroll
      for (int j4 = 0; j4 < 2; ++j4) {
        const float4 c4 = reinterpret_cast<const float4*>(Cv[h])[grp * 2 + j4];
        out[4 * j4] = c4.x; out[4 * j4 + 1] = c4.y; out[4 * j4 + 2] = c4.z; out[4 * j4 + 3] = c4.w;
      }
    };
    read_cc(0, cc[0]);
    read_cc(1, cc[1]);
    if constexpr (XC > 0) {  // fetches while the coefficients are on their way from LDS
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < XC; ++e) load_row(ifetch, XC0 + e, dst.v[XC0 + e]);
    }
    float acc[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] = h == 0 ? a.e[r] : 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int jj = 0; jj < KH; ++jj) {
      if (jj % S2 == 0 && jj / S2 < PR2) {
        // the multiply-adds so far stay ahead of this fetch (instruction selection would otherwise issue the
        // step's fetches in one burst while the coefficients are still on their way from LDS)
        if (jj > 0) asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));
        __builtin_amdgcn_sched_barrier(0);
        load_row(ifetch, U0 + jj / S2, dst.v[U0 + jj / S2]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[r] = fmaf(-cc[jj / 8][jj % 8], cur.v[jj].e[r], acc[r]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float sum = acc[r] + Lanes::partner(acc[r]);
      a.e[r] = keep[r] ? sum : 0.f;
    }
  };

  auto step_at = [&](int s) { return block_of(s < nb ? s : nb - 1); };  // fetches past the end repeat the last step
  Regs ra, rb, rc;
#pragma unroll
  for (int jj = 0; jj < KH; ++jj) load_row(step_at(0), jj, ra.v[jj]);
  load_t(step_at(0), ra);
#pragma unroll
  for (int jj = 0; jj < KH; ++jj) load_row(step_at(1), jj, rb.v[jj]);
  load_t(step_at(1), rb);
  int s = 0;
  for (; s + 2 < nb; s += 3) {
    apply_step(block_of(s), ra, step_at(s + 2), rc);
    apply_step(block_of(s + 1), rb, step_at(s + 3), ra);
    apply_step(block_of(s + 2), rc, step_at(s + 4), rb);
  }
  if (s < nb) {
    apply_step(block_of(s), ra, step_at(s + 2), rc);
    if (s + 1 < nb) apply_step(block_of(s + 1), rb, step_at(s + 3), ra);
  }
  if constexpr (SPLIT) {
    // the next launch on this workspace counts on from here (the partner read the counter before its first hand-off,
    // and this workgroup has received the partner's last one)
    if (half == 0 && tid == 0) __builtin_amdgcn_raw_buffer_store_b32(tag0 + steps_done, xdesc, 1024u, 0, 16);
    if (gave_up && lane == 0) __hip_atomic_store(&g_wait_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (ok) {
    // each lane of a pair stores two of the chunk's four elements
    const float o0 = h ? a.e[2] : a.e[0], o1 = h ? a.e[3] : a.e[1];
    if (!UNAL || x0 + 2 * h < (unsigned)d) p.out[(size_t)(x0 + 2 * h) * m + col] = o0;
    if (!UNAL || x0 + 2 * h + 1 < (unsigned)d) p.out[(size_t)(x0 + 2 * h + 1) * m + col] = o1;
  }
}

// Blocks of more than 16 rows (smaller ones would mostly fetch repeated rows in a 32-row step).
static bool chain_pair_serves(const ChainArgs& a) { return a.d <= 1024 && a.k > 16; }

template <int NW, int SUB, int P1, int RL, int XA, int XC, bool PAD = false, bool UNAL = false>
static int launch_chain_pair(const ChainArgs& args, hipStream_t stream) {
  ChainArgs a = args;
  a.sub = (args.k + 31) / 32;
  a.nb = args.nb * a.sub;
  if (!chain_pair_serves(a) || a.d > 128 * NW || (SUB > 0 && SUB != a.sub) || (!PAD && (a.k % 32 != 0 || a.kp != a.k)) ||
      32 * a.sub > a.kp || (!UNAL && a.d % 4 != 0))
    return FASTH_EINVAL;
  const int side = a.ds_out ? (a.ds_rows + NW - 1) / NW : 0;
  static const std::string name = variant_name("chain_pair_kernel", {NW, SUB, P1, RL, XA, XC, PAD, UNAL});
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, name.c_str());
  hipLaunchKernelGGL((chain_pair_kernel<NW, SUB, P1, RL, XA, XC, PAD, UNAL>), dim3(a.m + side), dim3(64 * NW), 0, stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

// Two workgroups per column (SPLIT above): 1024 < d <= 2048, whole 32-row steps, at most kSplitPairMaxCols columns
// so that every workgroup of the launch has a compute unit of its own and no half waits for a partner that has not
// started. (Shapes that chain_team_kernel takes never get here: the launcher asks it first.)
static bool chain_uses_split_pair(const ChainArgs& a) { return a.xch != nullptr && split_pair_serves(a.d, a.m, a.k); }

template <int SUB>
static int launch_chain_split_pair(const ChainArgs& args, hipStream_t stream) {
  ChainArgs a = args;
  a.sub = a.k / 32;
  a.nb = args.nb * a.sub;
  if (!chain_uses_split_pair(a) || SUB != a.sub || a.kp != a.k) return FASTH_EINVAL;
  static const std::string name = variant_name("chain_pair_kernel", {8, SUB, 4, 4, 3, 2, 0, 0, 1});
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, name.c_str());
  hipLaunchKernelGGL((chain_pair_kernel<8, SUB, 4, 4, 3, 2, false, false, true>), dim3(16 * ((a.m + 7) / 8)), dim3(512), 0,
                     stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

}  // namespace fasth
