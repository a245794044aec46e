// Algorithm 1 Step 2 and Algorithm 2 Step 1 for few columns of 513 to 4096 elements: chain_team_kernel, in which a
// team of two to eight workgroups shares a column and a step takes 64 rows, and chain_team_wide_kernel, in which the
// parts are half as long and a step takes 128 rows.
// Included by fasth_chain.h (the library has a single translation unit).
#pragma once
#include <hip/hip_runtime.h>

#include "fasth_common.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// A per-column chain is bound by what ONE compute unit can fetch and multiply per step: 32 rows x 1024 elements fill
// its registers, and a chain of n / 32 such steps is n / 32 times that. With few columns most units idle. Here a
// column of d elements is shared by NP = ceil(d / 512) workgroups ("parts", 2 to 8) on different compute units; part j keeps
// elements [512 j, 512 j + 512) of the column for the whole chain and reads only those columns of V, so the same
// registers hold 64 rows per step and the chain has n / 64 sequential steps. What the parts owe each other is a
// step's 64 partial inner products, nothing else: every part forms C = op(T) B itself.
//
// Blocks of 64 rows. By Lemma 1 the product of two consecutive blocks of 32 reflections is a WY block of 64:
// I - V^T T V with the 64 x 64 factor T = (diag(S)/2 + striu(S))^-1, S = V V^T, whose diagonal 32 x 32 blocks are
// the two blocks' own factors. Because T is triangular, the coefficients C = op(T) V a of the rows applied first are
// those of the first block alone, and the others are the second block's coefficients for ITS input; so for a
// caller's k = 32 the update is applied in two halves, the state between them is the second block's input, and what
// is saved for the backward pass is exactly what the other chain kernels save. For k = 128 the diagonal 64 x 64
// blocks of the block's factor serve its two steps (as in the other kernels).
//
// Lanes. A wave holds 64 elements of the column, a lane one 16-byte chunk (lane & 15) and every fourth row of the
// step (rows 4 jj + q, q = lane >> 4, jj < 16): 16 rows x 4 elements per lane and register copy, three copies as in
// chain_pair_kernel (the rows of step s + 2 are fetched while step s is applied); 16 adjacent lanes fetch 256
// contiguous bytes of one row. The 16 partial inner products of a lane are summed over the 16 lanes of its row of
// lanes by a register-only butterfly, after which lane (q, c) holds the wave's sum for row 4 c + q, and over the
// waves through LDS. In the update each lane subtracts its 16 rows' terms and the four lanes of a chunk add their
// sums through two lane-half swaps in an order that gives all four the same bits.
//
// Hand-off. After the sum over its own waves, wave w of a part owns rows 8 w .. 8 w + 7 of the step: it writes their
// sums as 8-byte words {value, tag} into every other part's inbox in the workspace (one store), polls its own
// inbox for the other parts' words (one load per poll), adds the NP sums in the order of the parts (so that every
// part gets the same bits) and puts the totals into LDS for all waves. A word is valid once its tag equals the
// step's; inboxes alternate between two sets by step parity (a part cannot be more than one step ahead of the
// others); tags count on from launch to launch through a word per column that the factor kernels zero together with
// the inboxes, so no stale word ever carries a valid tag, also when a captured launch is replayed. Stores and loads
// are agent-scope (correct wherever the parts run); the launch maps a team to one XCD (workgroups b, b + 8, ...),
// the parts tell each other their XCC_ID before the chain starts, and if they agree the hand-offs use ordinary
// stores (which the XCD's L2 holds) and loads that skip only the compute unit's own cache. Every wait is bounded:
// after p.wait_limit polls a wave gives up for the rest of the launch, raises the library's status word and runs on
// with what it has, so the kernel always ends; fasth_wait_status() tells the host.
// ------------------------------------------------------------------------------------------

struct TeamRegs {
  Chunk<4> v[16];  // rows 4 jj + q of the step, this lane's chunk
};

// KMODE 0: caller's blocks of 32 rows, two per step; 1: blocks of 64; 2: blocks of 128, two steps per block. The factors
// are stored as 64 x 64 blocks in every case. The number of parts is p.parts.
template <int KMODE>
__global__ void __launch_bounds__(512) chain_team_kernel(ChainArgs p) {
  const int NP = p.parts;  // 2 .. 8: the parts' sums are added within a group of eight lanes
  constexpr int K = kTeamRows, KH = 16, NW = 8, LPT = 8, G = 8;
  constexpr int LDT = 64;  // the factors are stored as 64 x 64 blocks whatever the caller's block size
  // fetches of step s + 2 per lane: P1 during the first product, RL during the reduction, XA behind the hand-off,
  // XC next to the last barrier, the rest during the update
  constexpr int P1 = 4, RL = 4, XA = 3, XC = 2, PR2 = KH - P1 - RL - XA - XC;
  constexpr int S1 = KH / P1, S2 = KH / PR2, XA0 = P1 + RL, XC0 = XA0 + XA, U0 = XC0 + XC;
  __shared__ float Bpart[NW][K + 1];          // per wave: its sums for the 64 rows (padded: column reads below)
  __shared__ __align__(16) float Btot[K];     // the step's inner products, summed over waves and parts
  __shared__ __align__(16) float Cv[4][KH];   // [q][jj] = coefficient of row 4 jj + q
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = p.m, d = p.d;
  // workgroups b, b + 8, ... (one XCD) are the parts of column 8 (b / (8 NP)) + b % 8
  const int chain_wgs = 8 * NP * ((m + 7) / 8);
  if ((int)blockIdx.x >= chain_wgs) {  // workgroups beyond the chain's: the side product, on compute units the chain leaves idle
    const int row = ((int)blockIdx.x - chain_wgs) * NW + wave;
    if (row < p.ds_rows) dsigma_row(p.in, p.ds_z1, p.in_scale, p.ds_out, row, m, p.in_scale_mode);
    return;
  }
  const int part = (int)(blockIdx.x >> 3) % NP;
  const int col = (int)(blockIdx.x >> 3) / NP * 8 + (int)(blockIdx.x & 7);
  if (col >= m) return;
  const int q = lane >> 4;
  const unsigned x0w = (unsigned)part * kTeamSlice + (unsigned)wave * 64u + 4u * (unsigned)(lane & 15);
  const bool ok = x0w < (unsigned)d;
  const unsigned x0 = ok ? x0w : 0u;  // lanes beyond d fetch chunk 0 (valid memory) and keep their elements at zero
  const unsigned lane_off = (unsigned)q * (unsigned)d + x0;
  Chunk<4> a = load_column_chunk<4>(p, col, x0, ok);
  const int trow = tid / G, tg = tid % G;  // G threads share a row of op(T), LPT entries each
  const int ns = p.n / K;                  // steps of the chain
  auto step_of = [&](int s) { return p.transpose ? s : ns - 1 - s; };  // index of the s-th step applied
  auto step_at = [&](int s) { return step_of(s < ns ? s : ns - 1); };  // fetches past the end repeat the last step

  const BufferDesc xdesc = make_buffer(reinterpret_cast<const float*>(p.xch + (size_t)col * team_words_per_column(NP)),
                                       team_words_per_column(NP) * 4u);
  const unsigned tag0 = __builtin_amdgcn_raw_buffer_load_b32(xdesc, 0u, 0, 16);
  bool gave_up = false, same_xcd = false;
  // Do the parts run on one XCD, i.e. behind one L2? Each publishes its XCC_ID (agent-scope, tagged like a hand-off)
  // first thing and reads the others' once its first rows of V are on their way.
  const unsigned my_xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;
  const unsigned hs_tag = tag0 + 1u;
  if (tid == 0) {
    const u32x2 w = {my_xcc, hs_tag};
    __builtin_amdgcn_raw_buffer_store_b64(w, xdesc, 32u + (unsigned)part * 8u, 0, 16);
  }

  auto load_row = [&](int st, int jj, Chunk<4>& dst) {
    dst = load_chunk<4>(p.V + ((size_t)st * K + 4 * jj) * (size_t)d + lane_off);
  };
  float t[LPT];  // this thread's entries of its row of op(T) of the step being applied
  auto load_t = [&](int st) {
    const float* opT = p.transpose ? p.Tt : p.T;
    const float* Ts = opT + (size_t)st * LDT * LDT;
    const float4* src = reinterpret_cast<const float4*>(Ts + trow * LDT + LPT * tg);
    const float4 t0 = src[0], t1 = src[1];
    t[0] = t0.x; t[1] = t0.y; t[2] = t0.z; t[3] = t0.w; t[4] = t1.x; t[5] = t1.y; t[6] = t1.z; t[7] = t1.w;
  };
  // Sums of four values over the four lanes of a chunk (lane bits 4 and 5), the same bits in all four lanes. First each
  // lane ends up with the complete sum of ONE of the values (halving twice: three lane-half swaps and three
  // additions instead of eight and eight), then the four sums are passed round (three more swaps).
  auto chunk_sums = [&](float (&x)[4]) {
    const float s01 = swap32_sum(x[0], x[1]);  // lanes 0..31: x0 over bit 5, lanes 32..63: x1
    const float s23 = swap32_sum(x[2], x[3]);
    const float one = swap16_sum(s01, s23);    // rows of lanes 0 / 1 / 2 / 3 hold the sums of x0 / x2 / x1 / x3
    const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(one), __float_as_uint(one), false, false);
    // r[0]: what the even row of this pair of rows holds, r[1]: what the odd row holds
    const u32x2 u = __builtin_amdgcn_permlane32_swap(r[0], r[0], false, false);  // lower half's, upper half's
    const u32x2 w = __builtin_amdgcn_permlane32_swap(r[1], r[1], false, false);
    x[0] = __uint_as_float(u[0]); x[1] = __uint_as_float(u[1]);
    x[2] = __uint_as_float(w[0]); x[3] = __uint_as_float(w[1]);
  };
  auto save_input = [&](int block) {
    if (p.save_in && ok && q == 0) store_chunk<4>(p.save_in + ((size_t)block * m + col) * d + x0, a);
  };

  unsigned steps_done = 0;
  // Applies step st held in `cur` while fetching step sf (two steps on) into `dst`.
  auto apply_step = [&](int st, TeamRegs& cur, int sf, TeamRegs& dst) {
    load_t(st);
    // the input of the caller's block that this step starts with
    if constexpr (KMODE == 0) save_input(2 * st + (p.transpose ? 0 : 1));
    else if constexpr (KMODE == 1) save_input(st);
    else if ((st & 1) == (p.transpose ? 0 : 1)) save_input(st >> 1);
    float pj[KH];
#pragma unroll
    for (int jj = 0; jj < KH; ++jj) {
      if (jj % S1 == 0 && jj / S1 < P1) {
        load_row(sf, jj / S1, dst.v[jj / S1]);
        __builtin_amdgcn_sched_barrier(0);
      }
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) acc = fmaf(cur.v[jj].e[r], a.e[r], acc);
      pj[jj] = acc;
    }
    auto prefetch = [&](int tt) {
      if (tt % 4 == 0 && tt / 4 < RL) {
        __builtin_amdgcn_sched_barrier(0);
        load_row(sf, P1 + tt / 4, dst.v[P1 + tt / 4]);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // sum over the 16 lanes of this row of lanes: 16 values, four lane bits; lane (q, c) ends with row 4 c + q
    reduce_stage<KH, 16, 8, 0>(pj, lane, prefetch);
    reduce_stage<KH, 8, 4, 8>(pj, lane, prefetch);
    reduce_stage<KH, 4, 2, 12>(pj, lane, prefetch);
    reduce_stage<KH, 2, 1, 14>(pj, lane, prefetch);
    Bpart[wave][4 * (lane & 15) + q] = pj[0];
    lds_barrier();
    {
      // wave w owns rows 8 w .. 8 w + 7: lane l takes wave (l & 7)'s sum for row 8 w + (l >> 3)
      const int row = 8 * wave + (lane >> 3), j = lane & 7;
      float b = group_sum<8>(Bpart[j][row]);
      const unsigned tag = tag0 + 1u + steps_done, par = steps_done & 1u;
      // lane j < NP of each group stands for part j: its own sum, or what part j sends
      const bool other = j < NP && j != part;
      if (other) {
        const u32x2 w = {__builtin_bit_cast(unsigned, b), tag};
        const unsigned to = (unsigned)kTeamHeadBytes + ((((unsigned)j * 2u + par) * NP + (unsigned)part) * K + (unsigned)row) * 8u;
        if (same_xcd) __builtin_amdgcn_raw_buffer_store_b64(w, xdesc, to, 0, 0);
        else __builtin_amdgcn_raw_buffer_store_b64(w, xdesc, to, 0, 16);
      }
      unsigned got = 0u;  // zero once a wait has given up
      if (!gave_up) {
        // lanes that stand for no other part read the word of one that does (and ignore its value)
        const unsigned src = other ? (unsigned)j : (part == 0 ? 1u : 0u);
        const unsigned from = (unsigned)kTeamHeadBytes + ((((unsigned)part * 2u + par) * NP + src) * K + (unsigned)row) * 8u;
        int polls = 0;
        for (;;) {
          const u32x2 w = same_xcd ? __builtin_amdgcn_raw_buffer_load_b64(xdesc, from, 0, 2)
                                   : __builtin_amdgcn_raw_buffer_load_b64(xdesc, from, 0, 16);
          got = w.x;
          if (__all(w.y == tag)) break;
          if (polls++ >= p.wait_limit) { gave_up = true; break; }
          asm volatile("" ::: "memory");
        }
      }
      // Lane j < NP of a group holds part j's sum in EVERY part (its own, or what part j sent), the other lanes zero, so
      // the same tree of additions over the group gives every part the same bits.
      const float mine = other ? __builtin_bit_cast(float, got) : (j == part ? b : 0.f);
      const float total = group_sum<8>(mine);
      if (j == 0) Btot[row] = total;
    }
    {  // fetches behind the hand-off (before it, its polls would queue up behind them: loads return in order)
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < XA; ++e) load_row(sf, XA0 + e, dst.v[XA0 + e]);
      __builtin_amdgcn_sched_barrier(0);
    }
    lds_barrier();
    {
      const float4 b0 = reinterpret_cast<const float4*>(Btot)[2 * tg], b1 = reinterpret_cast<const float4*>(Btot)[2 * tg + 1];
      float c = t[0] * b0.x;
      c = fmaf(t[1], b0.y, c); c = fmaf(t[2], b0.z, c); c = fmaf(t[3], b0.w, c);
      c = fmaf(t[4], b1.x, c); c = fmaf(t[5], b1.y, c); c = fmaf(t[6], b1.z, c); c = fmaf(t[7], b1.w, c);
      c = group_sum<G>(c);
      if (tg == 0) {
        Cv[trow & 3][trow >> 2] = c;
        if (p.save_c && part == 0) p.save_c[(size_t)col * p.n + (size_t)st * K + trow] = c;
      }
    }
    lds_barrier();
    float cc[KH];
#pragma unroll
    for (int j4 = 0; j4 < 4; ++j4) {
      const float4 c4 = reinterpret_cast<const float4*>(Cv[q])[j4];
      cc[4 * j4] = c4.x; cc[4 * j4 + 1] = c4.y; cc[4 * j4 + 2] = c4.z; cc[4 * j4 + 3] = c4.w;
    }
    {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < XC; ++e) load_row(sf, XC0 + e, dst.v[XC0 + e]);
    }
    // Rows 4 jj + q with jj < 8 are the step's rows 0 .. 31, the others its rows 32 .. 63. The half applied first is
    // the later block of the pair in the plain order, the earlier one in the transposed order.
    float acc[2][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { acc[0][r] = 0.f; acc[1][r] = 0.f; }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int jj = 0; jj < KH; ++jj) {
      if (jj % S2 == 0 && jj / S2 < PR2) {
        if (jj > 0) asm volatile("" : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[0][2]), "+v"(acc[0][3]));
        __builtin_amdgcn_sched_barrier(0);
        load_row(sf, U0 + jj / S2, dst.v[U0 + jj / S2]);
        __builtin_amdgcn_sched_barrier(0);
      }
      constexpr int kSplitAt = KMODE == 0 ? 8 : 16;
      const int hsel = jj < kSplitAt ? 0 : 1;
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[hsel][r] = fmaf(cc[jj], cur.v[jj].e[r], acc[hsel][r]);
    }
    if constexpr (KMODE == 0) {
      // The chain goes on from a minus both halves' terms at once; the state between the halves is only something to
      // save (the input of the pair's other block), formed beside the next step's first product.
      const int first = p.transpose ? 0 : 1;
      Chunk<4> mid = a;
      const bool want_mid = p.save_in != nullptr;
      float both[4], head[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        both[r] = acc[0][r] + acc[1][r];
        head[r] = first ? acc[1][r] : acc[0][r];
      }
      chunk_sums(both);
#pragma unroll
      for (int r = 0; r < 4; ++r) a.e[r] = ok ? a.e[r] - both[r] : 0.f;
      if (want_mid) {
        chunk_sums(head);
#pragma unroll
        for (int r = 0; r < 4; ++r) mid.e[r] -= head[r];
        if (ok && q == 0) store_chunk<4>(p.save_in + ((size_t)(2 * st + (p.transpose ? 1 : 0)) * m + col) * d + x0, mid);
      }
    } else {
      chunk_sums(acc[0]);
#pragma unroll
      for (int r = 0; r < 4; ++r) a.e[r] = ok ? a.e[r] - acc[0][r] : 0.f;
    }
    ++steps_done;
  };

  TeamRegs ra, rb, rc;
#pragma unroll
  for (int jj = 0; jj < KH; ++jj) load_row(step_at(0), jj, ra.v[jj]);
#pragma unroll
  for (int jj = 0; jj < KH; ++jj) load_row(step_at(1), jj, rb.v[jj]);
  {
    unsigned peer_xcc = my_xcc;
    const unsigned hs_from = 32u + (unsigned)(lane < NP ? lane : part) * 8u;  // every lane reads some part's word
    int polls = 0;
    for (;;) {
      const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(xdesc, hs_from, 0, 16);
      peer_xcc = w.x;
      if (__all(w.y == hs_tag)) break;
      if (polls++ >= p.wait_limit) { gave_up = true; break; }
      asm volatile("" ::: "memory");
    }
    same_xcd = !gave_up && __all(peer_xcc == my_xcc);
  }
  int s = 0;
  for (; s + 2 < ns; s += 3) {
    apply_step(step_of(s), ra, step_at(s + 2), rc);
    apply_step(step_of(s + 1), rb, step_at(s + 3), ra);
    apply_step(step_of(s + 2), rc, step_at(s + 4), rb);
  }
  if (s < ns) {
    apply_step(step_of(s), ra, step_at(s + 2), rc);
    if (s + 1 < ns) apply_step(step_of(s + 1), rb, step_at(s + 3), ra);
  }
  // the next launch on this workspace counts on from here (every part read the counter before its first hand-off,
  // and this part has received the others' last one)
  if (part == 0 && tid == 0) __builtin_amdgcn_raw_buffer_store_b32(tag0 + steps_done, xdesc, 0u, 0, 16);
  if (gave_up && lane == 0) __hip_atomic_store(&g_wait_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (ok) {
    // each of the four lanes of a chunk stores one of its elements
    const float o = q == 0 ? a.e[0] : q == 1 ? a.e[1] : q == 2 ? a.e[2] : a.e[3];
    p.out[(size_t)(x0 + q) * m + col] = o;
  }
}

// ------------------------------------------------------------------------------------------
// chain_team_wide_kernel: the same team of workgroups per column with 256 elements of the column per part and steps
// of 128 rows, so that a chain has n / 128 sequential steps (and hand-offs). A step joins two blocks a, b of 64 rows
// (the caller's, halves of the caller's blocks of 128, or merged pairs of the caller's blocks of 32: the factor
// kernel builds 64 x 64 factors for all of them). With B_a = V_a x, B_b = V_b x from ONE pass over the step's rows and
// one hand-off, the block applied first (b in the plain order) has C_b = op(T_b) B_b, and the other sees the input
// x - V_b^T C_b, i.e. C_a = op(T_a) (B_a - S C_b) with S = V_a V_b^T, which the factor kernel forms beside the factors
// (Lemma 1 with the product of the two factors left unformed: three 64 x 64 products per step, the same data as the
// merged factor of 128 rows, and no 128 x 128 inverse to build). The update is one pass again.
// Lanes: a wave holds 32 elements of the column, a lane one 16-byte chunk (lane & 7) and sixteen consecutive rows of
// the step (rows 16 q + jj, q = lane >> 3, jj < 16): the same 16 rows x 4 elements per lane and register copy, and
// all of a lane's rows belong to one of the caller's blocks. The butterfly over the 8 lanes of a row of lanes leaves
// two sums per lane (rows 16 q + 2 c and the next); wave w owns rows 16 w .. 16 w + 15 of the step in the hand-off,
// whose words are 16 bytes {sum, tag, sum, tag}. In the update the eight lanes of a chunk add their terms in three
// exchanges (lane bits 3, 4, 5); where an exchange crosses from one caller's block to the next it is a step of a
// prefix sum instead, so the states between the blocks cost no exchange of their own.
// The step's three 64 x 64 matrices (48 KiB) do not fit in registers beside three copies of the rows: they are
// fetched straight into LDS at the start of the step (stored by the factor kernel in the order in which the threads
// read them: thread 16 g + c takes entries 4 c .. 4 c + 3 of rows 2 g and 2 g + 1), and are there when the hand-off ends.
// ------------------------------------------------------------------------------------------
typedef __attribute__((address_space(1))) const void global_cvoid;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kWideBpartLd = kWideRows + 1;
constexpr int kWideMatFloats = 3 * 64 * 64;  // op(T) of the block applied first, op(S), op(T) of the other
constexpr size_t kWideLdsFloats = (size_t)kWideMatFloats + 8 * kWideBpartLd + kWideRows + kWideRows;
static_assert((kWideMatFloats + 8 * kWideBpartLd) % 4 == 0, "16-byte reads of the totals");

// KMODE 0: caller's blocks of 32 rows, four per step; 1: blocks of 64, two per step; 2: blocks of 128.
template <int KMODE>
__global__ void __launch_bounds__(512) chain_team_wide_kernel(ChainArgs p) {
  const int NP = p.parts;  // 2 .. 8
  constexpr int K = kWideRows, KH = 16, NW = 8, NSUB = KMODE == 0 ? 4 : KMODE == 1 ? 2 : 1;
  constexpr int P1 = 4, RL = 4, XA = 3, XC = 2, PR2 = KH - P1 - RL - XA - XC;
  constexpr int S1 = KH / P1, S2 = KH / PR2, XA0 = P1 + RL, XC0 = XA0 + XA, U0 = XC0 + XC;
  extern __shared__ __align__(16) float smem[];
  float* Ts = smem;                         // the step's three matrices, each [2][512] groups of four entries
  float* Bpart = Ts + kWideMatFloats;                // per wave: its sums for the 128 rows, [NW][kWideBpartLd]
  float* Btot = Bpart + NW * kWideBpartLd;  // the step's inner products, summed over waves and parts
  float* Cv = Btot + K;                     // the step's coefficients
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = p.m, d = p.d;
  const int chain_wgs = 8 * NP * ((m + 7) / 8);
  if ((int)blockIdx.x >= chain_wgs) {  // the side product, on compute units the chain leaves idle
    const int row = ((int)blockIdx.x - chain_wgs) * NW + wave;
    if (row < p.ds_rows) dsigma_row(p.in, p.ds_z1, p.in_scale, p.ds_out, row, m, p.in_scale_mode);
    return;
  }
  const int part = (int)(blockIdx.x >> 3) % NP;
  const int col = (int)(blockIdx.x >> 3) / NP * 8 + (int)(blockIdx.x & 7);
  if (col >= m) return;
  const int q = lane >> 3;
  const unsigned x0w = (unsigned)part * kWideSlice + (unsigned)wave * 32u + 4u * (unsigned)(lane & 7);
  const bool ok = x0w < (unsigned)d;
  const unsigned x0 = ok ? x0w : 0u;
  const unsigned lane_off = 16u * (unsigned)q * (unsigned)d + x0;
  Chunk<4> a = load_column_chunk<4>(p, col, x0, ok);
  const int ns = p.n / K;
  auto step_of = [&](int s) { return p.transpose ? s : ns - 1 - s; };
  auto step_at = [&](int s) { return step_of(s < ns ? s : ns - 1); };

  const BufferDesc xdesc = make_buffer(reinterpret_cast<const float*>(p.xch + (size_t)col * team_wide_words_per_column(NP)),
                                       team_wide_words_per_column(NP) * 4u);
  const unsigned tag0 = __builtin_amdgcn_raw_buffer_load_b32(xdesc, 0u, 0, 16);
  bool gave_up = false, same_xcd = false;
  const unsigned my_xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;
  const unsigned hs_tag = tag0 + 1u;
  if (tid == 0) {
    const u32x2 w = {my_xcc, hs_tag};
    __builtin_amdgcn_raw_buffer_store_b64(w, xdesc, 32u + (unsigned)part * 8u, 0, 16);
  }

  auto load_row = [&](int st, int jj, Chunk<4>& dst) {
    dst = load_chunk<4>(p.V + ((size_t)st * K + jj) * (size_t)d + lane_off);
  };
  // The step's matrices, straight into LDS: group e of this wave's threads is 1 KiB in a row, in memory and in LDS.
  // Blocks a = 2 st (rows 0 .. 63 of the step) and b = 2 st + 1; b is applied first in the plain order, a in the other.
  const int first = p.transpose ? 0 : 1;
  auto fetch_t = [&](int st) {
    const float* opT = p.transpose ? p.Tt : p.T;
    const float* src[3] = {opT + (size_t)(2 * st + first) * 4096, p.S + (size_t)st * 8192 + (p.transpose ? 4096 : 0),
                           opT + (size_t)(2 * st + 1 - first) * 4096};
#pragma unroll
    for (int mtx = 0; mtx < 3; ++mtx) {
#pragma unroll
      for (int e = 0; e < 2; ++e)
        __builtin_amdgcn_global_load_lds((global_cvoid*)(src[mtx] + ((size_t)e * 512 + tid) * 4),
                                         (lds_void*)(Ts + mtx * 4096 + ((size_t)e * 512 + 64 * wave) * 4), 16, 0, 0);
    }
  };
  // Row 2 (tid / 16) + b3 (b3: bit 3 of the lane) of a 64 x 64 matrix in LDS times 64 values in LDS: thread 16 g + c has
  // the terms of rows 2 g, 2 g + 1 from columns 4 c .. 4 c + 3, and the 16 lanes that share the rows add them.
  auto matvec = [&](const float* M, const float* vec) {
    const float4 b4v = reinterpret_cast<const float4*>(vec)[tid & 15];
    float ce[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const float4 t4 = reinterpret_cast<const float4*>(M)[e * 512 + tid];
      ce[e] = fmaf(t4.w, b4v.w, fmaf(t4.z, b4v.z, fmaf(t4.y, b4v.y, t4.x * b4v.x)));
    }
    NoHook nh;
    reduce_stage<2, 2, 8, 0>(ce, lane, nh);
    reduce_stage<2, 1, 4, 0>(ce, lane, nh);
    reduce_stage<2, 1, 2, 0>(ce, lane, nh);
    reduce_stage<2, 1, 1, 0>(ce, lane, nh);
    return ce[0];
  };
  const int mrow = 2 * (tid >> 4) + ((lane >> 3) & 1);  // the row whose product matvec leaves in this lane
  const bool mwrite = (lane & 7) == 0;
  auto save_input = [&](int block) {
    if (p.save_in && ok && q == 0) store_chunk<4>(p.save_in + ((size_t)block * m + col) * d + x0, a);
  };

  // Where this lane saves the state behind its own block of a step, the input of the block applied next (if there is
  // one in the step; of blocks of 64 rows two lanes hold the same sums): an offset from the step's first block.
  const int my_block = KMODE == 0 ? (lane >> 4) & 3 : KMODE == 1 ? (lane >> 5) & 1 : 0;
  const int next_block = p.transpose ? my_block + 1 : my_block - 1;
  const bool mid_ok = p.save_in != nullptr && ok && next_block >= 0 && next_block < NSUB && (KMODE == 0 || (lane & 16) == 0);
  const unsigned mid_off = mid_ok ? ((unsigned)next_block * (unsigned)m + (unsigned)col) * (unsigned)d + x0 + ((lane & 8) ? 2u : 0u) : 0u;

  unsigned steps_done = 0;
  auto apply_step = [&](int st, TeamRegs& cur, int sf, TeamRegs& dst) {
    // the input of the caller's block that this step starts with
    save_input(NSUB * st + (p.transpose ? 0 : NSUB - 1));
    float pj[KH];
#pragma unroll
    for (int jj = 0; jj < KH; ++jj) {
      if (jj % S1 == 0 && jj / S1 < P1) {
        load_row(sf, jj / S1, dst.v[jj / S1]);
        __builtin_amdgcn_sched_barrier(0);
      }
      float acc = 0.f;
#pragma unroll
      for (int r = 0; r < 4; ++r) acc = fmaf(cur.v[jj].e[r], a.e[r], acc);
      pj[jj] = acc;
    }
    __builtin_amdgcn_sched_barrier(0);
    fetch_t(st);
    __builtin_amdgcn_sched_barrier(0);
    auto prefetch = [&](int tt) {
      if (tt % 4 == 0 && tt / 4 < RL) {
        __builtin_amdgcn_sched_barrier(0);
        load_row(sf, P1 + tt / 4, dst.v[P1 + tt / 4]);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // sum over the 8 lanes of this row of lanes: 16 values, three lane bits; lane (q, c) ends with rows 16 q + 2 c
    // (pj[0]) and 16 q + 2 c + 1 (pj[1])
    reduce_stage<KH, 16, 4, 0>(pj, lane, prefetch);
    reduce_stage<KH, 8, 2, 8>(pj, lane, prefetch);
    reduce_stage<KH, 4, 1, 12>(pj, lane, prefetch);
    Bpart[wave * kWideBpartLd + 16 * q + 2 * (lane & 7)] = pj[0];
    Bpart[wave * kWideBpartLd + 16 * q + 2 * (lane & 7) + 1] = pj[1];
    // A barrier for LDS traffic written out, without a fence: behind a fence the compiler would wait for every fetch in
    // flight here, because the factor's fetch into LDS is one of them. Nothing reads the factor before the next barrier.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    {
      // wave w owns rows 16 w .. 16 w + 15: lane l takes wave (l & 7)'s sums for rows 16 w + (l >> 3) and that + 8
      const int rr = lane >> 3, j = lane & 7, row = 16 * wave + rr;
      const float b0 = group_sum<8>(Bpart[j * kWideBpartLd + row]);
      const float b1 = group_sum<8>(Bpart[j * kWideBpartLd + row + 8]);
      const unsigned tag = tag0 + 1u + steps_done, par = steps_done & 1u;
      const unsigned word = 8u * (unsigned)wave + (unsigned)rr;  // of the 64 that a part sends per step
      const bool other = j < NP && j != part;
      if (other) {
        const u32x4 w = {__builtin_bit_cast(unsigned, b0), tag, __builtin_bit_cast(unsigned, b1), tag};
        const unsigned to = (unsigned)kTeamHeadBytes + ((((unsigned)j * 2u + par) * NP + (unsigned)part) * 64u + word) * 16u;
        if (same_xcd) __builtin_amdgcn_raw_buffer_store_b128(w, xdesc, to, 0, 0);
        else __builtin_amdgcn_raw_buffer_store_b128(w, xdesc, to, 0, 16);
      }
      unsigned got0 = 0u, got1 = 0u;  // zero once a wait has given up
      if (!gave_up) {
        const unsigned src = other ? (unsigned)j : (part == 0 ? 1u : 0u);
        const unsigned from = (unsigned)kTeamHeadBytes + ((((unsigned)part * 2u + par) * NP + src) * 64u + word) * 16u;
        int polls = 0;
        for (;;) {
          // (the word is declared inside the loop and its entries copied out one by one on purpose)
          const u32x4 w = same_xcd ? __builtin_amdgcn_raw_buffer_load_b128(xdesc, from, 0, 2)
                                   : __builtin_amdgcn_raw_buffer_load_b128(xdesc, from, 0, 16);
          const unsigned t0 = w.y, t1 = w.w;
          got0 = w.x;
          got1 = w.z;
          if (__all(t0 == tag && t1 == tag)) break;
          if (polls++ >= p.wait_limit) { gave_up = true; break; }
          asm volatile("" ::: "memory");
        }
      }
      const float mine0 = other ? __builtin_bit_cast(float, got0) : (j == part ? b0 : 0.f);
      const float mine1 = other ? __builtin_bit_cast(float, got1) : (j == part ? b1 : 0.f);
      const float total0 = group_sum<8>(mine0), total1 = group_sum<8>(mine1);
      if (j == 0) {
        Btot[row] = total0;
        Btot[row + 8] = total1;
      }
    }
    // this wave's share of the factor is in LDS (the polls have waited for every earlier fetch; a wave that has given
    // up has not polled)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    {  // fetches behind the hand-off
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < XA; ++e) load_row(sf, XA0 + e, dst.v[XA0 + e]);
      __builtin_amdgcn_sched_barrier(0);
    }
    lds_barrier();
    {
      // C of the block applied first, the other block's inner products as that block's output leaves them, its C
      const int hf = 64 * first, hs = 64 - hf;  // the blocks' rows of the step
      const float c1 = matvec(Ts, Btot + hf);
      if (mwrite) {
        Cv[hf + mrow] = c1;
        if (p.save_c && part == 0) p.save_c[(size_t)col * p.n + (size_t)st * K + hf + mrow] = c1;
      }
      lds_barrier();
      const float u = matvec(Ts + 4096, Cv + hf);
      if (mwrite) Btot[hs + mrow] -= u;
      lds_barrier();
      const float c2 = matvec(Ts + 8192, Btot + hs);
      if (mwrite) {
        Cv[hs + mrow] = c2;
        if (p.save_c && part == 0) p.save_c[(size_t)col * p.n + (size_t)st * K + hs + mrow] = c2;
      }
    }
    lds_barrier();
    float cc[KH];
#pragma unroll
    for (int j4 = 0; j4 < 4; ++j4) {
      const float4 c4 = reinterpret_cast<const float4*>(Cv + 16 * q)[j4];
      cc[4 * j4] = c4.x; cc[4 * j4 + 1] = c4.y; cc[4 * j4 + 2] = c4.z; cc[4 * j4 + 3] = c4.w;
    }
    {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < XC; ++e) load_row(sf, XC0 + e, dst.v[XC0 + e]);
    }
    float x[4] = {0.f, 0.f, 0.f, 0.f};  // this lane's rows' terms: all of one caller's block
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int jj = 0; jj < KH; ++jj) {
      if (jj % S2 == 0 && jj / S2 < PR2) {
        if (jj > 0) asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]));
        __builtin_amdgcn_sched_barrier(0);
        load_row(sf, U0 + jj / S2, dst.v[U0 + jj / S2]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) x[r] = fmaf(cc[jj], cur.v[jj].e[r], x[r]);
    }
    // Sums over the eight lanes of a chunk (lane bits 3, 4, 5: 16, 32, 64 rows apart). First the lanes of a pair
    // share the work: the lane with bit 3 clear goes on with elements 0 and 1, the other with 2 and 3. The blocks
    // are applied last to first in the plain order, first to last in the transposed order; where an exchange joins
    // two of the caller's blocks, the lanes of the block applied second add the other's sum and the others keep
    // their own, so that a lane ends with the terms of all blocks up to its own: `a` minus that is the input of the
    // block applied next, which is only something to save. The chain goes on from `a` minus all blocks' terms.
    const bool b3 = (lane & 8) != 0, b4 = (lane & 16) != 0, b5 = (lane & 32) != 0;
    const float y0 = (b3 ? x[2] : x[0]) + dpp_move<kDppRowRor8>(b3 ? x[0] : x[2]);
    const float y1 = (b3 ? x[3] : x[1]) + dpp_move<kDppRowRor8>(b3 ? x[1] : x[3]);
    const u32x2 r0 = __builtin_amdgcn_permlane16_swap(__float_as_uint(y0), __float_as_uint(y0), false, false);
    const u32x2 r1 = __builtin_amdgcn_permlane16_swap(__float_as_uint(y1), __float_as_uint(y1), false, false);
    const float s0 = __uint_as_float(r0[0]) + __uint_as_float(r0[1]);  // even row of lanes + odd row
    const float s1 = __uint_as_float(r1[0]) + __uint_as_float(r1[1]);
    float p0 = s0, p1 = s1;
    if constexpr (KMODE == 0) {
      const bool second = p.transpose ? b4 : !b4;
      p0 = second ? s0 : y0;
      p1 = second ? s1 : y1;
    }
    const u32x2 h0 = __builtin_amdgcn_permlane32_swap(__float_as_uint(s0), __float_as_uint(s0), false, false);
    const u32x2 h1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(s1), __float_as_uint(s1), false, false);
    const float lo0 = __uint_as_float(h0[0]), hi0 = __uint_as_float(h0[1]);  // lower half of the wave, upper half
    const float lo1 = __uint_as_float(h1[0]), hi1 = __uint_as_float(h1[1]);
    const float t0 = lo0 + hi0, t1 = lo1 + hi1;
    if constexpr (KMODE <= 1) {
      const bool second = p.transpose ? b5 : !b5;
      if (second) {
        p0 += p.transpose ? lo0 : hi0;
        p1 += p.transpose ? lo1 : hi1;
      }
      if (mid_ok) {
        float a0 = a.e[0], a1 = a.e[1], a2 = a.e[2], a3 = a.e[3];
        asm("" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3));  // as values: the choices below stay choices between registers
        float2 mid;
        mid.x = (b3 ? a2 : a0) - p0;
        mid.y = (b3 ? a3 : a1) - p1;
        *reinterpret_cast<float2*>(p.save_in + (size_t)(NSUB * st) * m * d + mid_off) = mid;
      }
    }
    {
      const float g0 = dpp_move<kDppRowRor8>(t0), g1 = dpp_move<kDppRowRor8>(t1);  // the other pair of elements
      const float all[4] = {b3 ? g0 : t0, b3 ? g1 : t1, b3 ? t0 : g0, b3 ? t1 : g1};
#pragma unroll
      for (int r = 0; r < 4; ++r) a.e[r] = ok ? a.e[r] - all[r] : 0.f;
    }
    ++steps_done;
  };

  TeamRegs ra, rb, rc;
#pragma unroll
  for (int jj = 0; jj < KH; ++jj) load_row(step_at(0), jj, ra.v[jj]);
#pragma unroll
  for (int jj = 0; jj < KH; ++jj) load_row(step_at(1), jj, rb.v[jj]);
  {
    unsigned peer_xcc = my_xcc;
    const unsigned hs_from = 32u + (unsigned)(lane < NP ? lane : part) * 8u;
    int polls = 0;
    for (;;) {
      const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(xdesc, hs_from, 0, 16);
      peer_xcc = w.x;
      if (__all(w.y == hs_tag)) break;
      if (polls++ >= p.wait_limit) { gave_up = true; break; }
      asm volatile("" ::: "memory");
    }
    same_xcd = !gave_up && __all(peer_xcc == my_xcc);
  }
  int s = 0;
  for (; s + 2 < ns; s += 3) {
    apply_step(step_of(s), ra, step_at(s + 2), rc);
    apply_step(step_of(s + 1), rb, step_at(s + 3), ra);
    apply_step(step_of(s + 2), rc, step_at(s + 4), rb);
  }
  if (s < ns) {
    apply_step(step_of(s), ra, step_at(s + 2), rc);
    if (s + 1 < ns) apply_step(step_of(s + 1), rb, step_at(s + 3), ra);
  }
  if (part == 0 && tid == 0) __builtin_amdgcn_raw_buffer_store_b32(tag0 + steps_done, xdesc, 0u, 0, 16);
  if (gave_up && lane == 0) __hip_atomic_store(&g_wait_gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (ok && q < 4) {
    // four of the eight lanes of a chunk store one of its elements each
    const float o = q == 0 ? a.e[0] : q == 1 ? a.e[1] : q == 2 ? a.e[2] : a.e[3];
    p.out[(size_t)(x0 + q) * m + col] = o;
  }
}

static bool chain_uses_team_wide(const ChainArgs& a) { return a.xch != nullptr && team_wide_parts(a.d, a.n, a.m, a.k) > 0; }

static int launch_chain_team_wide(const ChainArgs& args, hipStream_t stream) {
  ChainArgs a = args;
  a.parts = team_wide_parts(a.d, a.n, a.m, a.k);
  if (a.parts == 0 || !a.xch) return FASTH_EINVAL;
  const int kmode = a.k == 32 ? 0 : a.k == 64 ? 1 : 2;
  const size_t lds = kWideLdsFloats * sizeof(float);
  int rc = kmode == 0 ? allow_lds(chain_team_wide_kernel<0>, lds)
         : kmode == 1 ? allow_lds(chain_team_wide_kernel<1>, lds) : allow_lds(chain_team_wide_kernel<2>, lds);
  if (rc != FASTH_OK) return rc;
  static const std::vector<std::string> names = [] {
    std::vector<std::string> v;
    for (int np = 2; np <= 8; ++np)
      for (int km = 0; km < 3; ++km)
        v.push_back(variant_name("chain_team_wide_kernel", {km}) + " (" + std::to_string(np) + " parts)");
    return v;
  }();
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, names[(a.parts - 2) * 3 + kmode].c_str());
  const int side = a.ds_out ? (a.ds_rows + 7) / 8 : 0;
  const dim3 grid(8 * a.parts * ((a.m + 7) / 8) + side), block(512);
  if (kmode == 0) hipLaunchKernelGGL(chain_team_wide_kernel<0>, grid, block, lds, stream, a);
  else if (kmode == 1) hipLaunchKernelGGL(chain_team_wide_kernel<1>, grid, block, lds, stream, a);
  else hipLaunchKernelGGL(chain_team_wide_kernel<2>, grid, block, lds, stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

static bool chain_uses_team(const ChainArgs& a) { return a.xch != nullptr && team_parts(a.d, a.n, a.m, a.k) > 0; }

static int launch_chain_team(const ChainArgs& args, hipStream_t stream) {
  ChainArgs a = args;
  a.parts = team_parts(a.d, a.n, a.m, a.k);
  if (a.parts == 0 || !a.xch) return FASTH_EINVAL;
  const int kmode = a.k == 32 ? 0 : a.k == 64 ? 1 : 2;
  // "chain_team_kernel<KMODE> (NP parts)" for NP = 2 .. 8
  static const std::vector<std::string> names = [] {
    std::vector<std::string> v;
    for (int np = 2; np <= 8; ++np)
      for (int km = 0; km < 3; ++km) v.push_back(variant_name("chain_team_kernel", {km}) + " (" + std::to_string(np) + " parts)");
    return v;
  }();
  prof::Scope ps_(FASTH_KERNEL_CHAIN, stream, names[(a.parts - 2) * 3 + kmode].c_str());
  const int side = a.ds_out ? (a.ds_rows + 7) / 8 : 0;  // a row of the side product per wave
  const dim3 grid(8 * a.parts * ((a.m + 7) / 8) + side), block(512);
  if (kmode == 0) hipLaunchKernelGGL(chain_team_kernel<0>, grid, block, 0, stream, a);
  else if (kmode == 1) hipLaunchKernelGGL(chain_team_kernel<1>, grid, block, 0, stream, a);
  else hipLaunchKernelGGL(chain_team_kernel<2>, grid, block, 0, stream, a);
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

}  // namespace fasth
