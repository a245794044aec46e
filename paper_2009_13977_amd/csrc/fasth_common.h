// Host-side shape bookkeeping, the workspace layout, error and timing helpers shared by the FastH kernels' launchers.
// Included by fasth.hip, the library's single translation unit.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

#include "fasth.h"
#include "fasth_device.h"

namespace fasth {

// ------------------------------------------------------------------------------------------
// Host-side shape bookkeeping
// ------------------------------------------------------------------------------------------

constexpr int kMaxBlock = 128;     // largest k: a k x k factor must fit in LDS with scratch
constexpr int kMaxD = 16384;       // general chain kernel: 1024 threads x 4 chunks of 4 elements
constexpr int kGramChunk = 128;    // columns of V per LDS tile in the Gram kernel
constexpr int kMaxGramSplit = 16;  // partial Gram matrices per block
constexpr int kComputeUnits = 256; // of the MI355X: launches of more workgroups than this run in rounds or share units
constexpr int kDvTile = 64;        // columns of dV per workgroup
constexpr int kDvMChunk = 32;      // mini-batch columns per LDS tile in the dV kernel

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int padded_block(int k) {
  int kp = 16;
  while (kp < k) kp *= 2;
  return kp;
}

struct Layout {
  int kp, nb, gram_split, dv_split;
  int kf, kpf, nbf;  // rows of a factor as stored (several of the caller's blocks when a team kernel merges them), padded; their number
  int team_wide;     // parts per column if chain_team_wide_kernel serves the shape (factors stored in its order), else 0
  int npair;         // pairs of blocks whose rows' product V_a V_b^T is formed beside the factors (chain_team_wide_kernel), else 0
  size_t off_T, off_S, off_Spart, off_ready, off_xch, off_saveA, off_saveCa, off_saveG, off_saveCg, off_dVpart, total;
  size_t xch_words;  // 32-bit words of the hand-off area between workgroups that share a column (0: none)
};

// Columns of 1025 to 2048 elements are shared by two workgroups (chain_pair_kernel's SPLIT form) while both have a
// compute unit of their own. Per column the workspace then holds 2 x 2 x 16 hand-off words of 16 bytes and a tag
// counter (padded to 256 bytes).
constexpr unsigned kSplitPairWords = (2 * 2 * 16 * 16 + 256) / 4;
constexpr int kSplitPairMaxCols = kComputeUnits / 2;
static bool split_pair_serves(int d, int m, int k) {
  return d > 1024 && d <= 2048 && d % 4 == 0 && (k == 32 || k == 64 || k == 128) && m <= kSplitPairMaxCols;
}
constexpr int kDefaultWaitLimit = 1 << 20;  // polls of a bounded wait between workgroups (a fraction of a second)

// chain_team_kernel: a team of two to eight workgroups per column, 512 elements each, steps of 64 rows. Parts per
// column for a shape it serves, else 0: 512 < d <= 4096 in whole 16-byte chunks, blocks of 32 (an even number of
// them: two are merged into a factor of 64 rows), 64 or 128 rows, and a compute unit for every workgroup of the
// launch, so that no part waits for one that has not started.
constexpr int kTeamRows = 64;        // rows of V per step
constexpr int kTeamSlice = 512;      // elements of the column per workgroup
constexpr int kTeamHeadBytes = 256;  // per column: [0] tag counter, [32 + 8 j] part j's XCC_ID word
constexpr unsigned team_words_per_column(int np) { return (unsigned)(kTeamHeadBytes + np * 2 * np * kTeamRows * 8) / 4u; }
#ifndef FASTH_TEAM_MIN_D
#define FASTH_TEAM_MIN_D (kTeamSlice + 1)
#endif
// A team's workgroups need a compute unit each, all at once: a part that waited for a unit would keep its partners
// polling until a whole chain elsewhere has ended. The launch places the parts of columns c, c + 8, ... on one XCD
// (32 of the 256 units), so what must fit is np workgroups for every eight columns begun.
static bool team_fits(int m, int np) { return 8 * np * ((m + 7) / 8) <= kComputeUnits; }
// chain_team_wide_kernel: the same with 256 elements of the column per workgroup and steps of 128 rows, for columns
// of FASTH_TEAM_WIDE_MIN_D to 2048 elements while every workgroup has a compute unit of its own: half as many
// sequential steps as with 64 rows. Such a step joins two blocks of 64 rows (the caller's, halves of the caller's
// blocks of 128, or merged pairs of the caller's blocks of 32) through their 64 x 64 factors and the product
// V_a V_b^T of their rows, which the factor kernel forms beside the factors. Its hand-off words are 16 bytes
// {sum, tag, sum, tag}. The matrices of such a shape are stored in the order in which the kernel's threads read them.
constexpr int kWideRows = 128;
constexpr int kWideSlice = 256;
constexpr unsigned team_wide_words_per_column(int np) { return (unsigned)(kTeamHeadBytes + np * 2 * np * (kWideRows / 2) * 16) / 4u; }
#ifndef FASTH_TEAM_WIDE_MIN_D
#define FASTH_TEAM_WIDE_MIN_D 513
#endif
static int team_wide_parts(int d, int n, int m, int k) {
  if (d < FASTH_TEAM_WIDE_MIN_D || d > 8 * kWideSlice || d % 4 != 0 || n % kWideRows != 0) return 0;
  if (!(k == 32 || k == 64 || k == 128)) return 0;
  const int np = (d + kWideSlice - 1) / kWideSlice;
  return team_fits(m, np) ? np : 0;
}
static int team_parts(int d, int n, int m, int k) {
  if (team_wide_parts(d, n, m, k)) return 0;
  if (d < FASTH_TEAM_MIN_D || d > 8 * kTeamSlice || d % 4 != 0) return 0;
  if (!(k == 64 || k == 128 || (k == 32 && n % 64 == 0))) return 0;
  const int np = (d + kTeamSlice - 1) / kTeamSlice;
  return team_fits(m, np) ? np : 0;
}

// chain_team_tile_kernel: tiles of 16 columns on the matrix cores, each shared by a team of ceil(d / 256) workgroups
// (2 to 4; ceil(d / 512) for d > 1024), steps of 64 rows (32 for d > 1024): for mini-batches of FASTH_TEAM_TILE_MIN_COLS columns and more (d > 512; ..._SHORT for
// shorter columns), as long as every
// workgroup has a compute unit on its team's XCD. Parts per tile for a shape it serves, else 0. Per tile the
// workspace holds a 256-byte head and, per receiving part, step parity and sending part, 512 hand-off words of 16 bytes.
#ifndef FASTH_TEAM_TILE_MIN_COLS
#define FASTH_TEAM_TILE_MIN_COLS 449        // d > 512: from here on it beats the per-column kernels' rounds (and chain_quad_kernel)
#endif
#ifndef FASTH_TEAM_TILE_MIN_COLS_LONG
#define FASTH_TEAM_TILE_MIN_COLS_LONG 640   // d > 1024 (parts of 512 elements, steps of 32 rows)
#endif
#ifndef FASTH_TEAM_TILE_MIN_COLS_SHORT
#define FASTH_TEAM_TILE_MIN_COLS_SHORT 897  // d <= 512 (two parts)
#endif
constexpr unsigned team_tile_words(int np) { return (unsigned)(kTeamHeadBytes + np * 2 * np * 512 * 16) / 4u; }
static int team_tile_parts(int d, int n, int m, int k) {
  if (m < (d > 1024 ? FASTH_TEAM_TILE_MIN_COLS_LONG : d > 512 ? FASTH_TEAM_TILE_MIN_COLS : FASTH_TEAM_TILE_MIN_COLS_SHORT) ||
      d <= 256 || d > 2048 || d % 4 != 0) return 0;
  // parts of 256 elements take 64 rows per step (blocks of 32 two at a time), parts of 512 (d > 1024) take 32
  if (!(k == 64 || k == 128 || (k == 32 && (d > 1024 || n % 64 == 0)))) return 0;
  if (team_wide_parts(d, n, m, k) || team_parts(d, n, m, k)) return 0;
  if ((size_t)d * m * sizeof(float) >= 0x80000000u || (size_t)n * d * sizeof(float) >= 0x80000000u) return 0;  // 32-bit byte offsets
  const int np = d > 1024 ? (d + 511) / 512 : (d + 255) / 256;
  return np >= 2 && team_fits((m + 15) / 16, np) ? np : 0;
}

// The dV kernel has one workgroup per (64-column tile of dV, block). When that is too few to fill the chip and the
// mini-batch is wide (a short, narrow V against many columns: a 1 x 1 convolution with few channels), the
// mini-batch is split over up to 32 workgroups whose partial sums meet in a buffer of the workspace.
static int dv_minibatch_split(int d, int n, int m, int k) {
  const int wgs = ((d + kDvTile - 1) / kDvTile) * (n / k);
  if (wgs >= 128 || m < 256) return 1;
  // a split needs every block's matrix Z formed beforehand from the coefficient matrices, which the kernel that does
  // it addresses with 32-bit byte offsets
  if ((size_t)m * n * sizeof(float) >= 0x80000000u) return 1;
  int split = 256 / wgs;
  if (split > m / 128) split = m / 128;
  if (split > 32) split = 32;
  return split < 1 ? 1 : split;
}

// Blocks of up to 32 rows are factored by one workgroup each; blocks of 64 rows only while d is short, because one
// workgroup per block then streams 64 d floats alone (measured: d = 256 18.0 -> 13.6 us, d = 1024 19.5 -> 21.5 us,
// d = 2048 23 -> 34 us against a Gram product split over d).
#ifndef FASTH_FUSED64_MAX_D
#define FASTH_FUSED64_MAX_D 512
#endif
static bool factor_is_fused(int kp, int d) { return kp <= 32 || (kp == 64 && d <= FASTH_FUSED64_MAX_D); }

#ifndef FASTH_GRAM_SPLIT_128
#define FASTH_GRAM_SPLIT_128 8
#endif
// shared = false: the layout without any kernel in which workgroups share columns (no hand-off area, the caller's own
// block size for the factors), for a caller whose room for factors is limited.
static Layout make_layout(int d, int n, int m, int k, bool shared = true) {
  Layout L;
  L.kp = padded_block(k);
  L.nb = n / k;
  const int team = shared ? team_parts(d, n, m, k) : 0, wide = shared ? team_wide_parts(d, n, m, k) : 0;
  const int ttile = shared ? team_tile_parts(d, n, m, k) : 0;
  // The kernels in which workgroups share columns take 64 rows (32: the shared tiles at d > 1024) of factor per step
  // whatever the caller's block size: two blocks of 32 merged by Lemma 1, or the diagonal blocks of a larger block's
  // factor, which are the factors of its row groups; so only those are built.
  L.kf = wide || team ? 64 : ttile ? (d <= 1024 ? 64 : 32) : k;
  L.team_wide = wide;
  L.npair = wide ? n / kWideRows : 0;
  L.kpf = padded_block(L.kf);
  L.nbf = n / L.kf;
  int split = (d + kGramChunk - 1) / kGramChunk;
  L.gram_split = split > kMaxGramSplit ? kMaxGramSplit : split;
  // factors of 128 rows: the workgroup that adds the partial matrices fetches four of them per trip to memory
  if (L.kpf == 128 && L.gram_split > FASTH_GRAM_SPLIT_128) L.gram_split = FASTH_GRAM_SPLIT_128;
  size_t off = 256;  // header, reserved
  auto take = [&](size_t floats) {
    size_t o = off;
    off = align_up(off + floats * sizeof(float), 256);
    return o;
  };
  L.off_T = take(2 * (size_t)L.nbf * L.kpf * L.kpf);  // the factors and, behind them, their transposes
  // partial Gram matrices (later the dV kernel's per-block matrices Z, nb kp^2 floats, which they always cover) and,
  // where the Gram product is split over workgroups, an 8-byte "ready" word per partial matrix
  L.off_Spart = take((size_t)(L.nbf + L.npair) * L.gram_split * L.kpf * L.kpf);
  L.off_ready = take(factor_is_fused(L.kpf, d) ? 0 : (size_t)(L.nbf + L.npair) * L.gram_split * 2);
  L.off_S = take(2 * (size_t)L.npair * L.kpf * L.kpf);  // per pair V_a V_b^T and its transpose
  L.xch_words = wide ? (size_t)m * team_wide_words_per_column(wide)
              : team ? (size_t)m * team_words_per_column(team)
              : ttile ? (size_t)((m + 15) / 16) * team_tile_words(ttile)
              : shared && split_pair_serves(d, m, k) ? (size_t)m * kSplitPairWords : 0;
  L.off_xch = take(L.xch_words);
  L.off_saveA = take((size_t)L.nb * m * d);
  L.off_saveCa = take((size_t)m * n);
  L.off_saveG = take((size_t)L.nb * m * d);
  L.off_saveCg = take((size_t)m * n);
  L.dv_split = dv_minibatch_split(d, n, m, k);
  L.off_dVpart = take(L.dv_split > 1 ? (size_t)L.dv_split * n * d : 0);
  L.total = off;
  return L;
}

static int check_shape(const fasth_shape* s) {
  if (!s) return FASTH_EINVAL;
  if (s->d < 1 || s->n < 1 || s->m < 1 || s->k < 1) return FASTH_EINVAL;
  if (s->n % s->k != 0) return FASTH_EINVAL;
  if (s->transpose != 0 && s->transpose != 1) return FASTH_EINVAL;
  if (s->k > kMaxBlock || s->d > kMaxD || s->m > 65535) return FASTH_EUNSUPPORTED;
  if (s->n / s->k > 65535) return FASTH_EUNSUPPORTED;  // blocks are a grid dimension of the factor and dV launches
  return FASTH_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Text of the last HIP error a call of this thread ran into, for fasth_strerror(FASTH_EHIP).
static thread_local char g_hip_error_text[192] = "";
static int note_hip_error(hipError_t e, const char* what) {
  snprintf(g_hip_error_text, sizeof(g_hip_error_text), "HIP runtime call or kernel launch failed: %s (%s)",
           hipGetErrorString(e), what);
  return FASTH_EHIP;
}

#define FASTH_HIP(call)                                    \
  do {                                                     \
    hipError_t e_ = (call);                                \
    if (e_ != hipSuccess) return note_hip_error(e_, #call); \
  } while (0)

// Optional per-kernel timing for benchmarks: a pair of HIP events around every launch.
// "kernel<a, b, c>": the instantiation a launcher picked, as a profiler prints it.
static std::string variant_name(const char* base, std::initializer_list<int> args) {
  std::string s(base);
  s += "<";
  bool first = true;
  for (int a : args) {
    if (!first) s += ", ";
    s += std::to_string(a);
    first = false;
  }
  return s + ">";
}

namespace prof {
struct Rec { int id; hipEvent_t beg, end; };
constexpr size_t kMaxRecords = 1u << 16;  // launches recorded between two collects; later ones go untimed
static bool enabled = false;
static std::vector<Rec> recs;
static std::vector<hipEvent_t> pool;
static const char* variant[FASTH_KERNEL_COUNT] = {};  // instantiation last launched per slot while enabled
static hipEvent_t get_event() {
  if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
struct Scope {
  Rec r{-1, nullptr, nullptr};
  hipStream_t st;
  Scope(int id, hipStream_t s, const char* name = nullptr) : st(s) {
    if (!enabled) return;
    if (name && id >= 0 && id < FASTH_KERNEL_COUNT) variant[id] = name;
    if (recs.size() >= kMaxRecords) return;
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

// Kernels that ask for more than 64 KiB of dynamic LDS must be allowed to, once per kernel and device; the size
// granted so far is remembered per kernel (a small table under a mutex) so that the timed path makes no such call.
struct LdsGrant { const void* kernel; int device; size_t bytes; };
static std::vector<LdsGrant> g_lds_grants;
static std::mutex g_lds_mutex;

template <typename K>
static int allow_lds(K kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return FASTH_OK;
  const void* fn = reinterpret_cast<const void*>(kernel);
  int dev = 0;
  FASTH_HIP(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(g_lds_mutex);
  for (LdsGrant& g : g_lds_grants) {
    if (g.kernel == fn && g.device == dev) {
      if (g.bytes >= bytes) return FASTH_OK;
      FASTH_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
      g.bytes = bytes;
      return FASTH_OK;
    }
  }
  FASTH_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  g_lds_grants.push_back(LdsGrant{fn, dev, bytes});
  return FASTH_OK;
}

}  // namespace fasth
