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
//   factor_fused_kernel  Algorithm 1 Step 1, one workgroup per block (block sizes up to 32; 64 for short vectors)
//   team_factor_kernel   Algorithm 1 Step 1 with a block's Gram product split over workgroups (MFMA); also the products
//                        V_a V_b^T of consecutive blocks' rows for the chain kernel that joins two blocks per step
//   chain_*_kernel       Algorithm 1 Step 2 / Algorithm 2 Step 1: the sequential block chain: per column of X
//                        (pair, pipe, general), a team of workgroups per column (team, team_wide), or 4 / 16 columns per
//                        workgroup on the matrix cores (quad, tile)
//   dv_kernel            Algorithm 2 Step 2 as dense products per block (MFMA)
//   seq_*                the one-reflection-at-a-time comparison
//   dsigma_kernel        the diagonal step of the SVD layer
// The kernels live in fasth_factor.h, fasth_chain.h (+ fasth_chain_team.h, fasth_chain_pair.h, fasth_chain_quad.h,
// fasth_chain_tile.h), fasth_dv.h and fasth_sequential.h (helpers in fasth_common.h and fasth_device.h); this file holds
// the host drivers and the C entry points.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdint>
#include <mutex>
#include <type_traits>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "fasth.h"
#include "fasth_device.h"
#include "fasth_common.h"
#include "fasth_factor.h"
#include "fasth_chain.h"
#include "fasth_dv.h"
#include "fasth_sequential.h"
#include "fasth_peaks.h"

namespace fasth {


// ------------------------------------------------------------------------------------------
// Host drivers
// ------------------------------------------------------------------------------------------

// Polls after which a kernel's wait for another workgroup gives up (fasth_set_wait_limit).
static std::atomic<int> g_wait_limit{kDefaultWaitLimit};
static int wait_limit() { return g_wait_limit.load(std::memory_order_relaxed); }

struct Product {  // one Householder product bound to its slice of a workspace
  int d, n, m, k;
  Layout L;
  char* ws;
  float* T() const { return reinterpret_cast<float*>(ws + L.off_T); }
  float* Spart() const { return reinterpret_cast<float*>(ws + L.off_Spart); }
  unsigned* xch() const { return L.xch_words ? reinterpret_cast<unsigned*>(ws + L.off_xch) : nullptr; }
  float* saveA() const { return reinterpret_cast<float*>(ws + L.off_saveA); }
  float* saveCa() const { return reinterpret_cast<float*>(ws + L.off_saveCa); }
  float* saveG() const { return reinterpret_cast<float*>(ws + L.off_saveG); }
  float* saveCg() const { return reinterpret_cast<float*>(ws + L.off_saveCg); }
};

static Product bind(int d, int n, int m, int k, void* ws, bool shared = true) {
  Product P;
  P.d = d; P.n = n; P.m = m; P.k = k;
  P.L = make_layout(d, n, m, k, shared);
  P.ws = static_cast<char*>(ws);
  return P;
}

static int launch_factor_fused(const FactorPair& fp, int count, int kp, bool vec4, hipStream_t stream) {
  static const std::string names[6] = {variant_name("factor_fused_kernel", {1, 4}), variant_name("factor_fused_kernel", {2, 4}),
                                       variant_name("factor_fused_kernel", {4, 4}), variant_name("factor_fused_kernel", {1, 1}),
                                       variant_name("factor_fused_kernel", {2, 1}), variant_name("factor_fused_kernel", {4, 1})};
  prof::Scope ps_(FASTH_KERNEL_FACTOR, stream, names[(vec4 ? 0 : 3) + (kp == 16 ? 0 : kp == 32 ? 1 : 2)].c_str());
  const dim3 grid(count == 2 && fp.nb[1] > fp.nb[0] ? fp.nb[1] : fp.nb[0], count), block(512);
  if (vec4) {
    if (kp == 16) hipLaunchKernelGGL((factor_fused_kernel<1, 4>), grid, block, 0, stream, fp);
    else if (kp == 32) hipLaunchKernelGGL((factor_fused_kernel<2, 4>), grid, block, 0, stream, fp);
    else hipLaunchKernelGGL((factor_fused_kernel<4, 4>), grid, block, 0, stream, fp);
  } else {
    if (kp == 16) hipLaunchKernelGGL((factor_fused_kernel<1, 1>), grid, block, 0, stream, fp);
    else if (kp == 32) hipLaunchKernelGGL((factor_fused_kernel<2, 1>), grid, block, 0, stream, fp);
    else hipLaunchKernelGGL((factor_fused_kernel<4, 1>), grid, block, 0, stream, fp);
  }
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

static void set_factor_slot(FactorPair& fp, int slot, const Product& P, const float* V) {
  fp.V[slot] = V; fp.T[slot] = P.T(); fp.d[slot] = P.d; fp.k[slot] = P.L.kf; fp.nb[slot] = P.L.nbf;
  fp.xch[slot] = P.xch(); fp.xch_words[slot] = (unsigned)P.L.xch_words;
}

static std::atomic<unsigned long long> g_launch_id{0x9e3779b97f4a7c15ull};  // a new value per launch, never 0

static TeamFactorArgs team_factor_args(const Product& P, const float* V) {
  TeamFactorArgs a;
  a.V = V; a.Spart = P.Spart(); a.T = P.T();
  a.ready = reinterpret_cast<unsigned long long*>(P.ws + P.L.off_ready);
  a.launch_id = g_launch_id.fetch_add(0x9e3779b97f4a7c15ull, std::memory_order_relaxed);
  if (a.launch_id == 0) a.launch_id = 1;
  a.d = P.d; a.k = P.L.kf; a.kp = P.L.kpf; a.split = P.L.gram_split; a.wait_limit = wait_limit();
  a.xch = P.xch(); a.xch_words = (unsigned)P.L.xch_words;
  a.S = reinterpret_cast<float*>(P.ws + P.L.off_S); a.nblocks = P.L.nbf; a.npair = P.L.npair;
  return a;
}

// Blocks of 64 or 128 rows (the caller's, or pairs of blocks of 32 merged for the team chain kernel): the Gram
// product split over d, the block's first workgroup inverts. `count` products of the same shape in one launch.
static int launch_team_factor(const TeamFactorPair& pair, int count, int nbf, hipStream_t stream) {
  const TeamFactorArgs& a = pair.a[0];
  // (a pair's workgroups stage the rows of two blocks)
  const size_t lds = std::max(sizeof(float) * (size_t)(a.npair > 0 ? 2 : 1) * a.kp * (kGramChunk + 4), t_build_lds(a.kp));
  const bool vec4 = a.d % 4 == 0;
  int rc = FASTH_OK;
  if (a.kp == 64) rc = vec4 ? allow_lds(team_factor_kernel<4, 64>, lds) : allow_lds(team_factor_kernel<1, 64>, lds);
  else rc = vec4 ? allow_lds(team_factor_kernel<4, 128>, lds) : allow_lds(team_factor_kernel<1, 128>, lds);
  if (rc != FASTH_OK) return rc;
  static const std::string names[4] = {variant_name("team_factor_kernel", {4, 64}), variant_name("team_factor_kernel", {1, 64}),
                                       variant_name("team_factor_kernel", {4, 128}), variant_name("team_factor_kernel", {1, 128})};
  prof::Scope ps_(FASTH_KERNEL_TEAM_FACTOR, stream, names[(a.kp == 64 ? 0 : 2) + (vec4 ? 0 : 1)].c_str());
  const dim3 grid(a.split, nbf + a.npair, count), block(8 * a.kp);
  if (a.kp == 64) {
    if (vec4) hipLaunchKernelGGL((team_factor_kernel<4, 64>), grid, block, lds, stream, pair);
    else hipLaunchKernelGGL((team_factor_kernel<1, 64>), grid, block, lds, stream, pair);
  } else {
    if (vec4) hipLaunchKernelGGL((team_factor_kernel<4, 128>), grid, block, lds, stream, pair);
    else hipLaunchKernelGGL((team_factor_kernel<1, 128>), grid, block, lds, stream, pair);
  }
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

static int build_factors(const Product& P, const float* V, hipStream_t stream) {
  const int kp = P.L.kpf;
  if (factor_is_fused(kp, P.d)) {
    FactorPair fp;
    set_factor_slot(fp, 0, P, V);
    set_factor_slot(fp, 1, P, V);  // unused
    return launch_factor_fused(fp, 1, kp, P.d % 4 == 0, stream);
  }
  TeamFactorPair pair;
  pair.a[0] = team_factor_args(P, V);
  pair.a[1] = pair.a[0];  // unused
  return launch_team_factor(pair, 1, P.L.nbf, stream);
}

// Factors of two products (independent of each other) in one launch when both take the fused
// kernel with the same template arguments; otherwise one after the other.
static int build_factors_pair(const Product& P0, const float* V0, const Product& P1, const float* V1,
                              hipStream_t stream) {
  if (factor_is_fused(P0.L.kpf, P0.d) && factor_is_fused(P1.L.kpf, P1.d) && P0.L.kpf == P1.L.kpf &&
      (P0.d % 4 == 0) == (P1.d % 4 == 0)) {
    FactorPair fp;
    set_factor_slot(fp, 0, P0, V0);
    set_factor_slot(fp, 1, P1, V1);
    return launch_factor_fused(fp, 2, P0.L.kpf, P0.d % 4 == 0, stream);
  }
  if (!factor_is_fused(P0.L.kpf, P0.d) && P0.d == P1.d && P0.n == P1.n && P0.L.kf == P1.L.kf &&
      P0.L.gram_split == P1.L.gram_split && P0.L.npair == P1.L.npair) {
    TeamFactorPair pair;
    pair.a[0] = team_factor_args(P0, V0);
    pair.a[1] = team_factor_args(P1, V1);
    return launch_team_factor(pair, 2, P0.L.nbf, stream);
  }
  const int rc = build_factors(P0, V0, stream);
  return rc != FASTH_OK ? rc : build_factors(P1, V1, stream);
}

// A = H in (transpose = 0) or H^T in (transpose = 1); activation = true saves into the activation
// slots of the workspace, false into the gradient slots.
static int run_chain(const Product& P, const float* V, const float* in, float* out, int transpose, bool activation,
                     const float* in_scale, int in_scale_mode, hipStream_t stream, bool save = true,
                     const Product* factors = nullptr, int in_rows = -1, const float* ds_z1 = nullptr,
                     float* ds_out = nullptr, int ds_rows = 0) {
  // `factors`: the product of the same shape whose workspace holds the block factors (and the hand-off area that
  // was cleared when they were built), if not P's own
  const Product& F = factors ? *factors : P;
  ChainArgs a;
  a.V = V; a.T = F.T(); a.in = in; a.out = out;
  a.xch = F.xch(); a.wait_limit = wait_limit(); a.parts = 0;
  a.S = reinterpret_cast<const float*>(F.ws + F.L.off_S);
  a.Tt = a.T + (size_t)F.L.nbf * F.L.kpf * F.L.kpf;
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
  a.msplit = P.L.dv_split;
  a.cols_per_part = ((P.m + a.msplit - 1) / a.msplit + kDvMChunk - 1) / kDvMChunk * kDvMChunk;
  a.dVpart = reinterpret_cast<float*>(P.ws + P.L.off_dVpart);
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
  const DvArgs& a0 = pair.a[0];
  const int msplit = a0.msplit;  // the same for both products of a launch (run_dv_pair checks)
  const dim3 grid(xt, nb, count * msplit);
  // Many columns and blocks of 64 rows or more: Z of every block once, by a launch of its own (measured at
  // d = n = 1024, m = 4096: dV 374 -> 326 us at k = 64, 853 -> 545 us at k = 128, but 294 -> 309 us at k = 32, where
  // the rebuild is a fifth of the work). Same condition for both products of a pair: they share m and k.
  // A split mini-batch needs it too: no workgroup sees all columns.
  const bool z_fits = (size_t)a0.m * a0.n * sizeof(float) < kOob && a0.Z != nullptr &&
                      (count == 1 || (pair.a[1].m == a0.m && pair.a[1].k == a0.k && pair.a[1].Z != nullptr));
  if (msplit > 1 && !z_fits) return FASTH_EINVAL;  // dv_minibatch_split never chooses a split for such a shape
  const bool prez = z_fits && (msplit > 1 || (a0.k >= 64 && (size_t)a0.m * a0.k >= 32768));
  static const std::string names[16] = {
      variant_name("dv_kernel", {1, 1, 0}), variant_name("dv_kernel", {1, 1, 1}), variant_name("dv_kernel", {1, 4, 0}), variant_name("dv_kernel", {1, 4, 1}),
      variant_name("dv_kernel", {2, 1, 0}), variant_name("dv_kernel", {2, 1, 1}), variant_name("dv_kernel", {2, 4, 0}), variant_name("dv_kernel", {2, 4, 1}),
      variant_name("dv_kernel", {4, 1, 0}), variant_name("dv_kernel", {4, 1, 1}), variant_name("dv_kernel", {4, 4, 0}), variant_name("dv_kernel", {4, 4, 1}),
      variant_name("dv_kernel", {8, 1, 0}), variant_name("dv_kernel", {8, 1, 1}), variant_name("dv_kernel", {8, 4, 0}), variant_name("dv_kernel", {8, 4, 1})};
  prof::Scope ps_(FASTH_KERNEL_DV, stream,
                  names[(kp == 16 ? 0 : kp == 32 ? 4 : kp == 64 ? 8 : 12) + (vec4 ? 2 : 0) + (prez ? 1 : 0)].c_str());
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
  if (msplit > 1) {
    size_t nd = (size_t)a0.n * a0.d;
    if (count == 2) nd = std::max(nd, (size_t)pair.a[1].n * pair.a[1].d);
    hipLaunchKernelGGL(dv_sum_kernel, dim3((unsigned)((nd + 255) / 256), count), dim3(256), 0, stream, pair);
    FASTH_HIP(hipGetLastError());
  }
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
  if (P0.L.kp == P1.L.kp && (P0.d % 4 == 0) == (P1.d % 4 == 0) && P0.L.dv_split == P1.L.dv_split) {
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
// Scratch memory of fasth_forward_static: one array per GPU, part of the loaded code object, so the call
// needs no allocation. In host code the array's name is only a handle; its device address is looked up once
// per device and kept.
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[FASTH_STATIC_SCRATCH_BYTES];

namespace fasth {
constexpr int kMaxDevices = 64;
static void* scratch_addr[kMaxDevices] = {};
static std::mutex scratch_mutex;

static int static_scratch(void** out) {
  int dev = -1;
  FASTH_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return FASTH_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_addr[dev]) {
    void* p = nullptr;
    FASTH_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return FASTH_EHIP;
    scratch_addr[dev] = p;
  }
  *out = scratch_addr[dev];
  return FASTH_OK;
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
    case FASTH_EHIP: return g_hip_error_text[0] ? g_hip_error_text : "HIP runtime call or kernel launch failed";
    case FASTH_EUNSUPPORTED: return "shape outside the supported range";
    case FASTH_ETIMEOUT: return "a kernel's wait for another workgroup gave up: results since the last check are invalid";
    default: return "unknown error code";
  }
}

int fasth_set_wait_limit(int polls) {
  g_wait_limit.store(polls < 0 ? kDefaultWaitLimit : polls, std::memory_order_relaxed);
  return FASTH_OK;
}

int fasth_wait_status(void* stream) {
  FASTH_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  unsigned word = 0;
  FASTH_HIP(hipMemcpyFromSymbol(&word, HIP_SYMBOL(g_wait_gave_up), sizeof(word)));
  if (!word) return FASTH_OK;
  const unsigned zero = 0;
  FASTH_HIP(hipMemcpyToSymbol(HIP_SYMBOL(g_wait_gave_up), &zero, sizeof(zero)));
  return FASTH_ETIMEOUT;
}

const char* fasth_kernel_name(int id) {
  switch (id) {
    case FASTH_KERNEL_TEAM_FACTOR: return "team_factor_kernel";
    case FASTH_KERNEL_RESERVED: return "";
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

const char* fasth_profile_variant(int id) {
  if (id < 0 || id >= FASTH_KERNEL_COUNT || !prof::variant[id]) return "";
  return prof::variant[id];
}

int fasth_profile_enable(int on) {
  prof::enabled = on != 0;
  if (on)
    for (int i = 0; i < FASTH_KERNEL_COUNT; ++i) prof::variant[i] = nullptr;
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

int fasth_measure_peaks(void* buffer, size_t buffer_bytes, int repetitions, float* fp32_mfma_tflops,
                        float* hbm_read_gbs, float* hbm_copy_gbs, void* stream) {
  if (!buffer || !fp32_mfma_tflops || !hbm_read_gbs || !hbm_copy_gbs || repetitions < 1) return FASTH_EINVAL;
  if (!aligned16(buffer)) return FASTH_EALIGN;
  if (buffer_bytes < (size_t)(8u << 20)) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  FASTH_HIP(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return FASTH_EHIP; }
  float* fbuf = static_cast<float*>(buffer);
  const int wgs = 4 * kComputeUnits, iters = 4096;
  const size_t pieces = buffer_bytes / 16, half = pieces / 2;
  int rc = FASTH_OK;
  float best[3] = {0.f, 0.f, 0.f};
  for (int which = 0; which < 3 && rc == FASTH_OK; ++which) {
    for (int rep = 0; rep <= repetitions && rc == FASTH_OK; ++rep) {  // the first pass is not timed
      if (hipEventRecord(e0, st) != hipSuccess) { rc = FASTH_EHIP; break; }
      if (which == 0) hipLaunchKernelGGL(peak_mfma_kernel, dim3(wgs), dim3(256), 0, st, fbuf, iters);
      else if (which == 1) hipLaunchKernelGGL(peak_read_kernel, dim3(8 * kComputeUnits), dim3(256), 0, st, static_cast<const float4*>(buffer) + 4096, pieces - 4096, fbuf);
      else hipLaunchKernelGGL(peak_copy_kernel, dim3(8 * kComputeUnits), dim3(256), 0, st, static_cast<const float4*>(buffer), static_cast<float4*>(buffer) + half, half);
      float ms = 0.f;
      if (hipGetLastError() != hipSuccess || hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
          hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { rc = FASTH_EHIP; break; }
      if (rep == 0 || ms <= 0.f) continue;
      float rate;
      if (which == 0) rate = (float)((double)wgs * 4 * iters * kPeakMfmaPerIter * 2048.0 / (ms * 1e-3) / 1e12);
      else if (which == 1) rate = (float)((double)(pieces - 4096) * 16.0 / (ms * 1e-3) / 1e9);
      else rate = (float)((double)half * 32.0 / (ms * 1e-3) / 1e9);  // bytes read + bytes written
      if (rate > best[which]) best[which] = rate;
    }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != FASTH_OK) return rc;
  *fp32_mfma_tflops = best[0]; *hbm_read_gbs = best[1]; *hbm_copy_gbs = best[2];
  return FASTH_OK;
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

int fasth_forward_static(const fasth_shape* shape, const float* V, const float* X, float* A, void* stream) {
  int rc = check_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !X || !A) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(X) || !aligned16(A)) return FASTH_EALIGN;
  // only the regions Step 1 writes and Step 2 reads: nothing is saved for a backward pass
  // (where the kernels in which workgroups share columns would need more room than the array has, the layout without
  // them: no hand-off area and the caller's own block size, and the chain runs on the other kernels)
  bool shared = true;
  Layout L = make_layout(shape->d, shape->n, shape->m, shape->k, true);
  if (L.off_saveA > FASTH_STATIC_SCRATCH_BYTES) {
    shared = false;
    L = make_layout(shape->d, shape->n, shape->m, shape->k, false);
  }
  if (L.off_saveA > FASTH_STATIC_SCRATCH_BYTES) return FASTH_EUNSUPPORTED;
  void* ws = nullptr;
  if ((rc = static_scratch(&ws)) != FASTH_OK) return rc;
  const Product P = bind(shape->d, shape->n, shape->m, shape->k, ws, shared);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = build_factors(P, V, st)) != FASTH_OK) return rc;
  return run_chain(P, V, X, A, shape->transpose, true, nullptr, 0, st, false);
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
  return (size_t)shape->m * shape->n * shape->d * sizeof(float);
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
    prof::Scope ps_(FASTH_KERNEL_SEQ_FORWARD, st, "seq_forward_kernel");
    FASTH_SEQ_DISPATCH(seq_forward_kernel, per, dim3(shape->m), dim3(threads), st, V, X, A, shape->d, shape->n,
                       shape->m, shape->transpose);
  }
  FASTH_HIP(hipGetLastError());
  return FASTH_OK;
}

int fasth_sequential_backward(const fasth_shape* shape, const float* V, const float* A, const float* G, float* dV,
                              float* dX, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_seq_shape(shape);
  if (rc != FASTH_OK) return rc;
  if (!V || !A || !G || !dV || !dX || !workspace) return FASTH_EINVAL;
  if (!aligned16(V) || !aligned16(A) || !aligned16(G) || !aligned16(dV) || !aligned16(dX) || !aligned16(workspace))
    return FASTH_EALIGN;
  if (workspace_bytes < fasth_sequential_workspace_bytes(shape)) return FASTH_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int d = shape->d, n = shape->n, m = shape->m;
  float* dVpart = static_cast<float*>(workspace);
  const int threads = seq_threads(d), per = (d + threads - 1) / threads;
  {
    prof::Scope ps_(FASTH_KERNEL_SEQ_BACKWARD, st, "seq_backward_kernel");
    FASTH_SEQ_DISPATCH(seq_backward_kernel, per, dim3(m), dim3(threads), st, V, A, G, dVpart, dX, d, n, m,
                       shape->transpose);
  }
  FASTH_HIP(hipGetLastError());
  const size_t nd = (size_t)n * d;
  {
    prof::Scope ps_(FASTH_KERNEL_SEQ_REDUCE, st, "seq_reduce_kernel");
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
  return run_chain(Pout, Uv, Z1, Y, 0, true, sigma, mode, st, true, &Pin);
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
  if ((rc = run_chain(Pout, Uv, G, dZ2, 1, false, nullptr, 0, st, true, &Pin)) != FASTH_OK) return rc;
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
