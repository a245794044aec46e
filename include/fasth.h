/*
 * fasth.h - C ABI of the FastH library for AMD CDNA4 (gfx950).
 *
 * FastH (arXiv 2009.13977, Algorithms 1 and 2) computes A = H X and the
 * gradients of a loss wrt X and the Householder vectors, where
 * H = H_1 H_2 ... H_n and H_j = I - 2 v_j v_j^T / ||v_j||^2 (Eq. 1). The n
 * reflections are grouped into n/k blocks P_i of k consecutive reflections
 * (Eq. 2 with the block size k of Section 3.3 "Trade-off"); every block is
 * turned into a compact WY form in parallel (Lemma 1, Algorithm 1 Step 1) and
 * the blocks are then applied one after the other (Algorithm 1 Step 2).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * - All array arguments are DEVICE pointers to dense row-major fp32, at least
 *   16-byte aligned. Shapes/sizes are plain ints passed by value or in a
 *   struct that lives in HOST memory.
 * - V is [n][d]: row j-1 holds v_j. H_1 is the leftmost factor, so v_n is
 *   applied to X first (Section 2.2 "Multiplication").
 * - X, A, G, dX, Y are [d][m]: one sample per column (the paper's d x m).
 * - The caller owns every buffer including the workspace. The library never
 *   allocates or frees device memory and keeps no pointer after a call
 *   returns. Outputs are overwritten, not accumulated. Outputs must not alias
 *   inputs.
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   All work is enqueued on it; no entry point synchronises with the host.
 * - Return value: FASTH_OK (0) or a negative FASTH_E* code. Argument checks
 *   happen before any GPU call, so they can be exercised on a host without a
 *   GPU. A zero Householder vector makes Eq. 1 undefined; it is not detected
 *   and produces Inf/NaN in the outputs.
 */
#ifndef FASTH_H
#define FASTH_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  FASTH_OK = 0,
  FASTH_EINVAL = -1,       /* null pointer, non-positive size, k does not divide n */
  FASTH_EWORKSPACE = -2,   /* workspace smaller than *_workspace_bytes() */
  FASTH_EALIGN = -3,       /* a pointer is not 16-byte aligned */
  FASTH_EHIP = -4,         /* a HIP runtime call or kernel launch failed */
  FASTH_EUNSUPPORTED = -5, /* shape outside the supported range (see fasth_shape) */
  FASTH_ETIMEOUT = -6      /* fasth_wait_status: a kernel's wait for another workgroup gave up */
};

/* Problem shape. Supported range: 1 <= d <= 16384, 1 <= n, 1 <= m <= 65535,
 * 1 <= k <= 128 and k divides n (the paper assumes the block size divides
 * the number of reflections, Section 3.1). n need not equal d. */
typedef struct fasth_shape {
  int d;          /* length of each Householder vector = rows of X */
  int n;          /* number of reflections = rows of V */
  int m;          /* columns of X (mini-batch size) */
  int k;          /* reflections per WY block (Section 3.3) */
  int transpose;  /* 0: A = H X.  1: A = H^T X = H_n ... H_1 X */
} fasth_shape;

/* Human-readable text for a return code (static storage, never NULL). */
const char* fasth_strerror(int code);

/* Algorithm 1 Step 2 is sequential over the blocks, but the two products of a block can be shared between compute
 * units. With few columns of more than 512 elements (d <= 4096, a compute unit for every workgroup of the launch:
 * up to 128 columns at d <= 1024, 64 at d = 2048, 32 at d = 4096) two to eight workgroups share each column and hand each other
 * every step's partial inner products through the workspace (steps of 128 rows, two blocks of 64 joined, where d <= 2048,
 * n is a multiple of 128 and a workgroup per 256 elements fits; steps of 64 rows otherwise; with some hundred columns
 * (449 to 1024, up to 2048 at d <= 512) of 257 to 2048 elements two to four workgroups share each tile of 16 columns in
 * the same way), and the workgroup that
 * adds the partial matrices of a block's factor waits for the workgroups that form them: one workgroup waits for
 * another inside a kernel. Every such wait is
 * bounded: after a number of polls (about a million, a fraction of a second; the wait itself takes a fraction of
 * a microsecond) the waiting wave gives up, raises a status word on the GPU and runs on, so a kernel always ends,
 * but its outputs are then wrong. fasth_wait_status waits for `stream`, reads and clears that word and returns
 * FASTH_OK, or FASTH_ETIMEOUT if any kernel of this library gave up on this GPU since the last check (by any
 * caller: the word is one per GPU, not per workspace). A caller that never checks loses nothing but the report.
 * fasth_set_wait_limit sets the number of polls for launches enqueued from now on (process-wide; negative
 * restores the default; 0 makes every wait give up at its first unsuccessful poll, which is how the error path is
 * tested without a kernel that hangs). The kernels assume what HIP provides on this hardware: the workgroups of
 * one launch are started in the order of their indices, and a launch of at most as many workgroups as the GPU
 * has compute units runs them all at once. That holds for calls on one stream; kernels of OTHER streams that run at
 * the same time (this library's or anyone's) can take compute units that a team needs, and two such launches can
 * hold each other's units while both wait: the waits then give up and fasth_wait_status says so. Run these shapes
 * on one stream at a time. Two calls that use the same workspace must not overlap on the GPU
 * (this was already so for calls that save for a backward pass; for these shapes it also holds for fasth_apply
 * without saving). */
int fasth_wait_status(void* stream);
int fasth_set_wait_limit(int polls);

/* Bytes of device workspace fasth_forward / fasth_backward need for `shape`
 * (block factors T_i, partial Gram matrices, the saved block inputs A_{i+1}
 * of Algorithm 1's Remark, the saved gradients dL/dA_i of Algorithm 2 Step 1,
 * the small per-block coefficient vectors and, for a small V against a wide
 * mini-batch, partial sums of dV). Returns 0 if the shape is invalid or
 * unsupported. */
size_t fasth_workspace_bytes(const fasth_shape* shape);

/* Algorithm 1. A = H X (or H^T X). Step 1 builds, for every block i, the
 * k x k upper-triangular factor T_i with P_i = I - V_i^T T_i V_i (V_i = the
 * block's k rows of V); this is the WY form of Lemma 1 with Y = V_i^T and
 * W = V_i^T T_i / 2. Step 2 applies the blocks sequentially and saves the
 * input of every block in the workspace for fasth_backward. */
int fasth_forward(const fasth_shape* shape, const float* V, const float* X, float* A,
                  void* workspace, size_t workspace_bytes, void* stream);

/* The two steps of Algorithm 1 as separate calls, for the uses of Section 3.3 ("Recurrent Layers")
 * where one H is applied many times: fasth_prepare runs Step 1 (block factors into the workspace)
 * once; fasth_apply runs Step 2 only and may be called any number of times, with any X of the
 * shape's size, while V and the workspace are unchanged. With save_for_backward != 0 it also saves
 * the block inputs, so fasth_prepare + fasth_apply(save) is exactly fasth_forward; with 0 nothing
 * but A is written (inference). */
int fasth_prepare(const fasth_shape* shape, const float* V, void* workspace, size_t workspace_bytes,
                  void* stream);
int fasth_apply(const fasth_shape* shape, const float* V, const float* X, float* A,
                void* workspace, size_t workspace_bytes, int save_for_backward, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, serving loops that
 * forbid it, harnesses without an allocator): A = H X (or H^T X) exactly as fasth_forward computes it,
 * with the block factors in a fixed array of FASTH_STATIC_SCRATCH_BYTES that is part of the library's
 * GPU code (one copy per GPU, held until the process ends) instead of a caller's workspace. Nothing is
 * saved for a backward pass. The call allocates and frees nothing; its first use on a device looks up
 * the array's address. Shapes whose factors, partial Gram matrices and hand-off words need more than the array
 * holds (about 4 n kp (2 + min(16, ceil(d / 128))) bytes, kp = k rounded up to a power of two >= 16; for the
 * shapes of fasth_wait_status's comment kp = 64 whatever k, half as much again where a step takes 128 rows, and up
 * to 129 KiB more per column: 10 MiB at d = n = 2048, m = 64, 17.5 MiB at m = 32; where that is too much the call
 * does without those kernels and needs the first figure only) return FASTH_EUNSUPPORTED before any GPU call. Every call on one GPU uses the same array: calls that overlap
 * on one GPU (different streams or threads) race; calls on one stream do not. */
#define FASTH_STATIC_SCRATCH_BYTES (24u << 20)
int fasth_forward_static(const fasth_shape* shape, const float* V, const float* X, float* A, void* stream);

/* Algorithm 2. Given G = dL/dA [d][m], writes dX = dL/dX [d][m] and
 * dV [n][d] (row j-1 = dL/dv_j, summed over the m columns, Eq. 5). The
 * workspace must be exactly as the fasth_forward call with the same shape
 * and V left it. Step 1 (Eq. 3) is the sequential block chain on G; Step 2 is
 * evaluated per block as dense matrix products that equal the sum of Eq. 5
 * over the block's reflections. */
int fasth_backward(const fasth_shape* shape, const float* V, const float* G,
                   float* dV, float* dX, void* workspace, size_t workspace_bytes, void* stream);

/* Section 3.3 "Trade-off": the block size k trades total work against the number of sequential
 * steps, and the paper picks it by trying the candidates once on the hardware at hand. This call
 * times fasth_forward + fasth_backward (`repetitions` >= 1 timed passes after one untimed pass) for
 * every candidate block size and writes the fastest to *best_k and its milliseconds per pass to
 * *best_ms (may be NULL); both are HOST pointers. `candidates` is a HOST array of ncandidates block
 * sizes, or NULL for every divisor of n in [2, 128]. Candidates that do not divide n, are out of
 * range, or need more workspace than given are skipped; FASTH_EUNSUPPORTED if none is left.
 * shape->k is ignored. Unlike every other entry point this one waits for the stream (it reads
 * event times). On return A, dV, dX hold the results of the last candidate run, which do not
 * depend on k beyond rounding. */
int fasth_tune_block_size(const fasth_shape* shape, const int* candidates, int ncandidates, int repetitions,
                          const float* V, const float* X, const float* G, float* A, float* dV, float* dX,
                          void* workspace, size_t workspace_bytes, int* best_k, float* best_ms, void* stream);

/* The comparison the paper measures against (the one-reflection-at-a-time evaluation of Section 2.2):
 * the same A, dX and dV computed one reflection at a time on the GPU, n dependent inner products over d
 * forward and 2 n backward. shape->k is ignored. fasth_sequential_backward takes A, the product that
 * fasth_sequential_forward wrote for the same V and X: walking the reflections from the output side it
 * recovers each reflection's input from its output (Eq. 4), so it needs neither X nor a second forward
 * pass. Its workspace holds one Eq. 5 term per column and reflection (m n d floats), which a last kernel
 * sums over the columns in a fixed order. */
size_t fasth_sequential_workspace_bytes(const fasth_shape* shape);
int fasth_sequential_forward(const fasth_shape* shape, const float* V, const float* X, float* A,
                             void* stream);
int fasth_sequential_backward(const fasth_shape* shape, const float* V, const float* A, const float* G,
                              float* dV, float* dX, void* workspace, size_t workspace_bytes,
                              void* stream);

/* SVD-reparameterised layer (Section 2.2): W = U diag(sigma) V^T with
 * U = prod H(u_j) and V = prod H(v_j), each a product of n Householder
 * reflections of length d given as rows of Uv, Vv [n][d]; sigma is [d].
 * Table 1, row "Inverse": W^-1 = V diag(1/sigma) U^T. */
typedef struct fasth_svd_shape {
  int d, n, m, k;
} fasth_svd_shape;

size_t svd_layer_workspace_bytes(const fasth_svd_shape* shape);

/* Y = W X = U (sigma * (V^T X)). */
int svd_layer_apply(const fasth_svd_shape* shape, const float* Uv, const float* sigma,
                    const float* Vv, const float* X, float* Y,
                    void* workspace, size_t workspace_bytes, void* stream);
/* Y = W^-1 X = V ((U^T X) / sigma). sigma must be non-zero. */
int svd_layer_inverse_apply(const fasth_svd_shape* shape, const float* Uv, const float* sigma,
                            const float* Vv, const float* X, float* Y,
                            void* workspace, size_t workspace_bytes, void* stream);
/* Gradients of L with G = dL/dY, after the matching *_apply call on the same
 * workspace and arguments: dUv, dVv [n][d], dsigma [d], dX [d][m]. */
int svd_layer_apply_backward(const fasth_svd_shape* shape, const float* Uv, const float* sigma,
                             const float* Vv, const float* G,
                             float* dUv, float* dsigma, float* dVv, float* dX,
                             void* workspace, size_t workspace_bytes, void* stream);
int svd_layer_inverse_apply_backward(const fasth_svd_shape* shape, const float* Uv, const float* sigma,
                                     const float* Vv, const float* G,
                                     float* dUv, float* dsigma, float* dVv, float* dX,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* The symmetric forms of Table 1 (rows "Matrix Exponential" and "Cayley map"): with one orthogonal
 * factor U (n reflections, rows of Uv) and W = U diag(sigma) U^T,
 *   FASTH_DIAG_IDENTITY: Y = W X
 *   FASTH_DIAG_EXP:      Y = e^W X            = U diag(e^sigma) U^T X
 *   FASTH_DIAG_CAYLEY:   Y = (I - W)(I + W)^-1 X = U diag((1 - sigma)/(1 + sigma)) U^T X   (sigma != -1)
 * The block factors of U are built once and used by both products. The workspace has the size
 * svd_layer_workspace_bytes() returns. The backward call follows the apply call on the same workspace
 * and arguments and writes dUv [n][d] (both uses of U added), dsigma [d] and dX [d][m]. */
enum { FASTH_DIAG_IDENTITY = 0, FASTH_DIAG_EXP = 1, FASTH_DIAG_CAYLEY = 2 };
int svd_sym_apply(const fasth_svd_shape* shape, int function, const float* Uv, const float* sigma,
                  const float* X, float* Y, void* workspace, size_t workspace_bytes, void* stream);
int svd_sym_apply_backward(const fasth_svd_shape* shape, int function, const float* Uv, const float* sigma,
                           const float* G, float* dUv, float* dsigma, float* dX,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Section 3.3 "Rectangular Matrices": W [rows][cols] = U Sigma V^T with U = prod H(u_j) of size
 * rows x rows (Uv is [n_u][rows]), V = prod H(v_j) of size cols x cols (Vv is [n_v][cols]) and Sigma
 * rows x cols, zero except Sigma_ii = sigma[i] for i < min(rows, cols). X and dX are [cols][m]; Y and G
 * are [rows][m]; k must divide both n_u and n_v; each of (rows, n_u) and (cols, n_v) obeys the limits
 * of fasth_shape. Y = U (Sigma (V^T X)); the backward call follows the apply call on the same
 * workspace and arguments and writes dUv [n_u][rows], dsigma [min(rows, cols)], dVv [n_v][cols], dX. */
typedef struct fasth_rect_shape {
  int rows, cols, n_u, n_v, m, k;
} fasth_rect_shape;
size_t svd_rect_workspace_bytes(const fasth_rect_shape* shape);
int svd_rect_apply(const fasth_rect_shape* shape, const float* Uv, const float* sigma, const float* Vv,
                   const float* X, float* Y, void* workspace, size_t workspace_bytes, void* stream);
int svd_rect_apply_backward(const fasth_rect_shape* shape, const float* Uv, const float* sigma, const float* Vv,
                            const float* G, float* dUv, float* dsigma, float* dVv, float* dX,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Table 1, row "Determinant": *log_abs_det (one float in device memory) = sum_i log|sigma_i| =
 * log|det(U diag(sigma) V^T)|; if dsigma is not NULL it receives the gradient 1/sigma_i. */
int svd_layer_log_abs_det(int d, const float* sigma, float* log_abs_det, float* dsigma, void* stream);

/* Benchmark aid (not part of the method). While enabled, every kernel this library launches from
 * the calling process is bracketed by a pair of HIP events on its stream; fasth_profile_collect
 * waits for them, adds the elapsed milliseconds and the launch count per kernel into the two HOST
 * arrays of FASTH_KERNEL_COUNT entries, and forgets the records. The extra events perturb
 * end-to-end timing, so keep profiling off in regions that report throughput. The profiling state is
 * process-global and not thread-safe. (What else the library remembers between calls: which kernels it has
 * already allowed more than 64 KiB of LDS, under a lock; the wait limit and status word of fasth_wait_status;
 * a counter from which every factor launch with a split Gram product draws its number.) */
enum {
  FASTH_KERNEL_TEAM_FACTOR = 0,
  FASTH_KERNEL_RESERVED = 1, /* no kernel: its entries stay zero */
  FASTH_KERNEL_CHAIN = 2,
  FASTH_KERNEL_DV = 3,
  FASTH_KERNEL_SEQ_FORWARD = 4,
  FASTH_KERNEL_SEQ_BACKWARD = 5,
  FASTH_KERNEL_SEQ_REDUCE = 6,
  FASTH_KERNEL_DSIGMA = 7,
  FASTH_KERNEL_FACTOR = 8,
  FASTH_KERNEL_COUNT = 9
};
const char* fasth_kernel_name(int id);
int fasth_profile_enable(int on);
int fasth_profile_collect(float* ms, int* launches);
/* The instantiation ("kernel<template arguments>") last launched in slot `id` since profiling was switched
 * on; "" if none. At most 65536 launches are timed between two collects; later ones run untimed. */
const char* fasth_profile_variant(int id);

/* Benchmark aid: what this GPU delivers on the rooflines the kernels are priced against, from plain kernels of
 * known work: fp32 matrix instructions issued from registers on every compute unit (TFLOP/s), a streaming read
 * of `buffer` and a copy of its first half onto its second (GB/s; the copy counts bytes read plus bytes written).
 * `buffer` is caller-owned device memory of at least 8 MiB, overwritten; several hundred MiB make the figures
 * those of HBM rather than of the caches. Best of `repetitions` timed runs each, after one untimed run. The three
 * results are HOST pointers. Waits for the stream (it reads event times). */
int fasth_measure_peaks(void* buffer, size_t buffer_bytes, int repetitions, float* fp32_mfma_tflops,
                        float* hbm_read_gbs, float* hbm_copy_gbs, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTH_H */
