/*
 * libslim -- the per-linear-layer quantisation pass of SliM-LLM (salience-driven mixed-precision
 * group quantisation, arXiv 2405.14917) as hand-written gfx950 (MI355X) HIP kernels.
 *
 * Notation is the paper's (Sec. 3.1, Alg. 1):  W in R^{n x m} with n output rows and m input
 * channels; calibration activations are handed over as X in R^{m x t} (input channels x tokens);
 * beta = group size along the input dimension, k = m / beta groups; N = target average width;
 * allowed widths {N-1, N, N+1}.
 *
 * Conventions for every entry point
 *  - Pointers are DEVICE pointers unless the comment says "host".  All matrices are row-major with
 *    an explicit leading dimension counted in elements.  The caller owns every buffer passed in;
 *    the library's device workspace is either the caller's too (given to slim_create, sized with
 *    slim_workspace_query: then no entry point allocates) or an internal grow-only one that slim_destroy frees.
 *  - Work is enqueued on the HIP stream given to slim_create.  A call returns as soon as its work
 *    is enqueued, except where it has a host output (info, p_star, obj_curve, m_star, n_bad, loss_curve): those calls
 *    wait until that output has arrived (slim_hessian_inverse: until the factorisation is done, with
 *    the rest of its work still in flight).  p_star, obj_curve, m_star, n_bad and loss_curve may be NULL: the call then
 *    does not wait.  slim_gptq_quantize and slim_lwc_quantize read the widths back for validation (and kernel selection),
 *    the former behind work it has already enqueued: the one wait of the host inside a pass.
 *  - Return value: SLIM_OK or a negative slim_status.  No exceptions, no aborts.  After an error
 *    slim_last_error(ctx) describes it; on SLIM_ERR_INVALID_ARG / SLIM_ERR_UNSUPPORTED no output
 *    was touched (at most work on the library's own workspace has been launched).  The one exception are the two
 *    checks of slim_pack that depend on device data (a width outside the range, a capacity that is too small): they
 *    are made on the device while the call runs, and packed / gbits / row_off then hold no valid result.
 *  - Device pointers must be 16-byte aligned, leading dimensions of 16-bit matrices multiples
 *    of 8 elements.
 *  - Calls on one context must not overlap in time (one stream, one workspace).
 *  - Results are deterministic: the same inputs give the same bytes on every run.
 */
#ifndef SLIM_H
#define SLIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct slim_ctx slim_ctx;

typedef enum {
  SLIM_OK = 0,
  SLIM_ERR_INVALID_ARG = -1, /* bad size, null / misaligned pointer, inconsistent arguments   */
  SLIM_ERR_NOT_PD = -2,      /* H + lambda I is not positive definite                           */
  SLIM_ERR_ALLOC = -3,       /* the workspace could not be grown, or the caller's is too small   */
  SLIM_ERR_HIP = -4,         /* a HIP runtime call failed                                       */
  SLIM_ERR_UNSUPPORTED = -5  /* valid in the paper's terms but not built (dtype, mode, size)    */
} slim_status;

typedef enum { SLIM_F16 = 0, SLIM_BF16 = 1, SLIM_F32 = 2, SLIM_F64 = 3 } slim_dtype;

/* Mode switches for the points the paper leaves open; value 0 is the default everywhere. */
enum { SLIM_WEIGHT_MASK_MEAN = 0, SLIM_WEIGHT_UNIFORM = 1, SLIM_WEIGHT_ELEMENT = 2 };
enum { SLIM_Q1_SIGN = 0, SLIM_Q1_AFFINE = 1 };
enum { SLIM_SCOPE_BLOCK = 0, SLIM_SCOPE_ROW = 1 };
enum { SLIM_SAL_HINV_DIAG = 0, SLIM_SAL_CHOL_DIAG = 1 };
enum { SLIM_OBJ_KL = 0, SLIM_OBJ_MSE = 1 };

typedef struct slim_params {
  /* SQC loss weights (Eq. 5, Alg. 2 SQC lines 13-15):
   *   MASK_MEAN  L = L_s/|s| + L_us/|us|  (mean squared error of the 3-sigma salient part plus that
   *              of the rest; a part without elements contributes nothing),
   *   UNIFORM    L = L_s + L_us (Eq. 5 as printed),
   *   ELEMENT    L = sum_j delta_j e_j^2 with delta_j = w_j^2 / [H^-1]_jj^2 (Def. 1).             */
  int sqc_weight_mode;
  /* statistics of the 3-sigma rule (Sec. 3.3.2): over the whole current n x beta block, or per row */
  int mask_scope;
  /* width-1 groups: sign / mean-absolute-value quantiser of Eq. 2, or two-level Eq. 1              */
  int q1_mode;
  /* salience denominator: [H^-1]_jj (Def. 1) or U_jj (Alg. 2 SBA line 6 read literally)            */
  int sal_mode;
} slim_params;

/* Host only.  Fills *p with the defaults (all zero). */
void slim_default_params(slim_params* p);

/* Host only.  Writes the default SQC candidate grid tau_c = (1 - lambda) + c * (lambda / n),
 * c = 0 .. 2n-1, lambda = 0.1, n = 50 (Sec. 3.3.2; Alg. 2 SQC lines 3-4 and 8) into tau_host[0..cap)
 * and returns the number of candidates (100).  tau_host may be NULL to query the count. */
int slim_default_tau(double* tau_host, int cap);

/* Shape of a layer, for slim_workspace_query: n output rows, m input channels, group size beta, t_c tokens per
 * call of slim_hessian_accumulate, t_s tokens of the SBA objective, t_x tokens per call of slim_dequant_matmul.
 * A field that is 0 leaves out the entry points that need it. */
typedef struct slim_shape {
  int n, m, beta;
  int64_t t_c, t_s;
  int t_x;
  int lwc_steps;       /* steps of slim_lwc_quantize (0: that entry point is not used) */
} slim_shape;

/* Host only.  Bytes of device workspace that the entry points need for a layer of exactly this shape: the largest
 * requirement of any single entry point (calls on one context run one after the other and reuse the workspace).
 * num_cus: compute units of the device (the split of the Gram matrix and of the linear layer depend on it); 0 = 256.
 * For several shapes take the largest answer: the requirement is not monotone in the sizes (a small Gram matrix
 * is split into more token ranges). */
size_t slim_workspace_query(const slim_shape* shape, int num_cus);

/* Creates a context bound to `hip_stream` (a hipStream_t, may be NULL for the default stream) on
 * the current device.  Allocates small fixed device buffers (default tau grid, flags).
 *   workspace, workspace_bytes   device memory of the caller (256-byte aligned) that the entry points use as their
 *       workspace until slim_destroy: with it NO entry point calls hipMalloc or hipFree, and a call whose shape needs
 *       more than workspace_bytes returns SLIM_ERR_ALLOC without touching anything (slim_workspace_query gives the
 *       size).  workspace = NULL: the context keeps a workspace of its own that grows on demand (hipMalloc / hipFree and
 *       a stream synchronisation inside the first call of every larger shape) and is freed by slim_destroy. */
slim_status slim_create(slim_ctx** out, void* hip_stream, void* workspace, size_t workspace_bytes);
slim_status slim_destroy(slim_ctx* ctx);
const char* slim_last_error(const slim_ctx* ctx);
/* Bytes of device workspace currently held by the context (host only). */
size_t slim_workspace_bytes(const slim_ctx* ctx);

/* ---------------------------------------------------------------------------------------------
 * a1  Proxy Hessian (Eq. 3; Alg. 1 line 1).   G += X_c X_c^T  for one chunk of t_c tokens.
 *   X        m x t_c, F16 or BF16, tokens contiguous (ldx >= t_c), read only
 *   G        m x m fp32 raw Gram matrix, both triangles kept up to date; the caller zero-initialises
 *            it before the first chunk.  H = (2 / n_tokens) G is formed lazily by slim_hessian_inverse.
 *   n_tokens host, in/out: incremented by t_c
 * Products are exact (fp16 x fp16 in fp32), accumulation is fp32 in the matrix cores.
 * t_c may be any positive number (a ragged tail is zero-padded internally); m must be a multiple of 8.
 */
slim_status slim_hessian_accumulate(slim_ctx* ctx, const void* X, slim_dtype x_dtype, int m, int64_t t_c,
                                    int64_t ldx, float* G, int64_t ldg, int64_t* n_tokens);

/* ---------------------------------------------------------------------------------------------
 * a2  Damped inverse and its Cholesky factor (Def. 1; Alg. 1 line 2).
 *   H = (2 / n_tokens) G,  lambda = percdamp * mean(diag H),
 *   U = upper-triangular factor with (H + lambda I)^-1 = U^T U  (fp64, m x m; the strictly lower
 *       triangle is written as zero),  hinv_diag_j = [(H + lambda I)^-1]_jj = sum_i U_ij^2.
 *   info  host: 0 on success, otherwise the 1-based index of a column at which a non-positive pivot
 *         appeared; the call then returns SLIM_ERR_NOT_PD and U / hinv_diag hold no valid result.
 * Only the upper triangle of G is read.  All arithmetic after widening G is fp64.
 */
slim_status slim_hessian_inverse(slim_ctx* ctx, const float* G, int64_t ldg, int m, int64_t n_tokens,
                                 double percdamp, double* U, int64_t ldu, double* hinv_diag, int* info);

/* ---------------------------------------------------------------------------------------------
 * a3  Salience (Def. 1; Alg. 2 SBA line 6).
 *   col_sal_j   = sum_i w_ij^2 / d_j^2          (m values)
 *   group_sal_g = mean over the n x beta entries of group g of w_ij^2 / d_j^2   (k values)
 *   elem_sal    = optional n x m map (ld = m), may be NULL
 *   d_j = hinv_diag_j (SLIM_SAL_HINV_DIAG) or U_jj (SLIM_SAL_CHOL_DIAG).
 *   W is F16, BF16 or F32, n x m, read only.
 */
slim_status slim_salience(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                          const double* U, int64_t ldu, const double* hinv_diag, int sal_mode, int beta,
                          double* col_sal, double* group_sal, double* elem_sal);

/* ---------------------------------------------------------------------------------------------
 * a4  Salience-Determined Bit Allocation (Eq. 4; Alg. 2 SBA; App. C and D).
 *   Groups are ranked by group_sal (stable, ascending).  For p = 0 .. floor(k/2): the p least salient
 *   groups get N-1 bits, the p most salient N+1, the rest N; the original W is fake-quantised per
 *   (row, group) with the default parameters of Eq. 1 (Eq. 2 for width 1) and the objective is
 *   sum over the t_s tokens of KL(softmax(x W^T) || softmax(x W_p^T)), softmax over the n outputs.
 *   The smallest p attaining the minimum is kept.  objective = SLIM_OBJ_MSE replaces the KL divergence by the
 *   squared error of the same outputs, || x W^T - x W_p^T ||_F^2 (the loss of Eq. 3; the variant of App. D).
 *   X_s       m x t_s (F16/BF16), tokens contiguous, the calibration tokens used by the objective
 *   bits      device, k bytes: the chosen width of every group
 *   p_star    host, or NULL
 *   obj_curve host, floor(k/2)+1 doubles or NULL: the objective for every p
 *   N in 2..7 (widths N - 1 .. N + 1 within 1..8; the paper's settings are N = 2, 3 and, in App. G, 4).  All
 *   arithmetic is fp64.
 */
slim_status slim_sba_allocate(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                              const double* group_sal, int beta, int N, int objective, const void* X_s,
                              slim_dtype x_dtype, int64_t t_s, int64_t ldxs, const slim_params* params,
                              uint8_t* bits, int* p_star, double* obj_curve);

/* Optional first half of slim_sba_allocate (Eq. 4): everything of the objective that does not depend on the
 * ranking of the groups - the reference outputs x W^T and their softmax statistics, and the outputs of the weights
 * with every group at N bits - is computed and kept in the context's workspace.  It needs neither the Hessian nor
 * the salience, so a caller with a second context on a second stream can run it beside slim_hessian_inverse
 * (a chain of small kernels that leaves most of the chip idle; the products here leave some CUs to it).
 * Asynchronous, no host output.  The next call on this context must be slim_sba_allocate with the same W, X_s,
 * shapes, N, objective and params, which then only ranks, searches and finishes; with any other argument, or after
 * any other call on the context, slim_sba_allocate computes everything itself.  W and X_s must not change in
 * between.  The result of slim_sba_allocate is bit for bit the same either way. */
slim_status slim_sba_prepare(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw, int beta,
                             int N, int objective, const void* X_s, slim_dtype x_dtype, int64_t t_s, int64_t ldxs,
                             const slim_params* params);

/* ---------------------------------------------------------------------------------------------
 * a5 + a6  3-sigma mask and Salience-Weighted Quantizer Calibration on ONE n x beta block of
 * current weights (Sec. 3.3.2; Eq. 5; Alg. 1 line 8; Alg. 2 SQC).
 *   For every row: delta0, z from Eq. 1 on the row's beta values (z does not depend on tau); for each
 *   candidate c: delta = tau_c delta0, loss L_c = sum_j omega_j (w_j - w_hat_j)^2; first minimum wins.
 *   Width 1 with SLIM_Q1_SIGN: alpha = mean|w|, w_hat = tau_c alpha sign(w); reported as
 *   scale = 2 tau alpha, zero = 1/2, so that w_hat = scale * (q - zero) holds for every width.
 *   Wblk      n x beta fp64 (ldw >= beta)
 *   omega     optional n x beta fp64 (ld = beta) explicit loss weights; NULL = derive from params
 *   hinv_diag_blk  beta values of [H^-1]_jj for the block's columns, needed by SLIM_WEIGHT_ELEMENT only
 *   tau       ncand candidates (device), or NULL for the default grid (then ncand is ignored)
 *   scale, zero  n doubles each;  cand_idx  n ints or NULL
 *   beta in {32, 64, 128, 256, 512}; bits in 1..8.
 */
slim_status slim_sqc_calibrate(slim_ctx* ctx, const double* Wblk, int64_t ldw, int n, int beta, int bits,
                               const double* omega, const double* hinv_diag_blk, const slim_params* params,
                               const double* tau, int ncand, double* scale, double* zero, int* cand_idx);

/* ---------------------------------------------------------------------------------------------
 * a5 - a8  Main loop (Alg. 1 lines 5-13) with GPTQ's column-serial error compensation.
 *   For each group b (beta columns): mask + SQC on the current weights of the group; then column by
 *   column q = Q(w_c), w_hat = scale (q - zero), e = (w_c - w_hat) / U_cc, remaining columns of the
 *   group get w_j -= e U_cj; after the group all later columns get W[:, later] -= E_b U[b, later].
 *   W         n x m, F16/BF16/F32, read only; the working copy (fp64) lives in the workspace
 *   U         from slim_hessian_inverse (fp64, upper triangular, zero below the diagonal)
 *   bits      device, k bytes, every value in 1..8 (codes are bytes)
 *   beta        32, 64, 128, 256 or 512
 *   gptq_block  columns swept between two trailing updates: beta, or 128 for wider groups (groups wider than
 *               128 columns are always swept in 128-column blocks; the result does not depend on it)
 *   hinv_diag needed by SLIM_WEIGHT_ELEMENT only, else may be NULL
 *   codes     n x m bytes (ld = m);  scale, zero  n x k doubles (ld = k)
 *   What      optional dequantised weights n x m (ld = m) in what_dtype (F32 or F64), or NULL
 *   sum_e2    optional device double: sum of squares of all compensation errors e
 * All arithmetic is fp64, so that rounding decisions agree with a float64 reference.
 */
slim_status slim_gptq_quantize(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                               const double* U, int64_t ldu, const uint8_t* bits, int beta, int gptq_block,
                               const slim_params* params, const double* hinv_diag, const double* tau,
                               int ncand, uint8_t* codes, double* scale, double* zero, void* What,
                               slim_dtype what_dtype, double* sum_e2);

/* ---------------------------------------------------------------------------------------------
 * a9  Storage format (App. B.2).
 *   row_off[g] = sum_{g' < g} beta * bits[g'] / 32  (k+1 ints; row_off[k] = m_star)
 *   packed     m_star x n 32-bit words (ld = n): for group g and output row i the beta codes form a
 *              little-endian bit stream (element r at bits [r b, (r+1) b)) whose words occupy rows
 *              row_off[g] .. of column i.  No padding, no word mixes two widths.
 *   gbits      ceil(k/16) words: bits[g] - bit_base as a 2-bit value, 16 groups per word, least significant first
 *   bit_base   the width that the value 0 stands for.  A layer of target width N holds the widths N - 1, N, N + 1
 *              only (constraint of Eq. 4), so three of the four values are ever used: 1 for the targets 2 and 3 (widths 1..4);
 *              N - 2 above them (2 for the 4-bit setting of App. G, widths 3..5).  It belongs to the stored form:
 *              a reader needs the same value.
 *   packed_rows  capacity of `packed` in rows; if m_star exceeds it the call fails with
 *              SLIM_ERR_INVALID_ARG and writes nothing beyond the capacity
 *   m_star     host, or NULL: the call then does not wait for the stream and can report neither a width outside
 *              bit_base .. bit_base + 3 nor a capacity that is too small (it still writes nothing beyond the capacity); m_star is
 *              row_off[k]
 *   beta * b must be a multiple of 32 for every width in use (beta a multiple of 32); widths up to 8.
 */
slim_status slim_pack(slim_ctx* ctx, const uint8_t* codes, int n, int m, int64_t ldc, const uint8_t* bits,
                      int beta, int bit_base, uint32_t* packed, int64_t packed_rows, uint32_t* gbits,
                      int32_t* row_off, int* m_star);

/* ---------------------------------------------------------------------------------------------
 * a9  Zero points as packed integers (App. B.2: packed with one precision along the channel direction).
 *   zero      n x k doubles (ld = ldz), as slim_gptq_quantize writes them (device)
 *   zbits     width of a stored zero point, 2..16.  The stored value is 2 z (Eq. 1 gives integer zeros, the sign form of
 *             width 1 has z = 1/2); a layer of target width N has zeros up to 2^(N+1) - 1, so N + 2 bits hold them
 *   zpacked   k x ceil(n zbits / 32) words (ld = ldzp): for every group the n values form a little-endian bit stream
 *             along the output channels, element i at bits [i zbits, (i + 1) zbits)
 *   n_bad     host, or NULL (the call then does not wait): the number of zero points that are not a multiple of 1/2
 *             or do not fit (Eq. 1 does not bound the zero of a group whose weights all have one sign); they are stored
 *             as 0 or the largest value, whichever is nearer, and the layer should keep its zeros in floating point
 * slim_unpack_zeros is the inverse (z = stored value / 2, exact).
 */
slim_status slim_pack_zeros(slim_ctx* ctx, const double* zero, int n, int k, int64_t ldz, int zbits, uint32_t* zpacked,
                            int64_t ldzp, int* n_bad);
slim_status slim_unpack_zeros(slim_ctx* ctx, const uint32_t* zpacked, int64_t ldzp, int n, int k, int zbits,
                              double* zero, int64_t ldz);

/* ---------------------------------------------------------------------------------------------
 * n1  Linear layer on the stored form (App. B.2, inference; built from the list of next steps).
 *   Y[t][i] = sum_j X[t][j] * scale[i][g] * (q_ij - zero[i][g]),   g = j / beta   (Eq. 1),
 *   the codes q_ij decoded from packed / gbits / row_off exactly as slim_pack writes them.
 *   packed   m_star x n words (ld = ldp >= n);  gbits ceil(k/16) words;  row_off k+1 ints   (device)
 *   scale, zero   n x k doubles (ld = k), as written by slim_gptq_quantize (device); a zero that is a
 *            multiple of 1/2 within +-511 takes the fastest path (Eq. 1 gives integers, the sign form of width 1 uses
 *            1/2); any other finite zero (Eq. 1 does not bound -round(w_min / delta0): a group of one sign with a narrow
 *            range has a large one) is accepted and costs that (row, group) a correction term
 *   X        t_x x m, F16 or BF16, channels contiguous (ldx >= m);  t_x >= 1 tokens, taken 16 at a time (the kernels are
 *            built for the few tokens of a decoding step; more tokens are a sequence of such steps on the stream)
 *   Y        t_x x n fp32 (ldy >= n), overwritten
 *   beta     a multiple of 32 that divides m
 *   bit_base as given to slim_pack; 1 or 2 (widths up to 5), anything else is SLIM_ERR_UNSUPPORTED.  A group whose
 *            width (from gbits and bit_base) disagrees with its rows, (row_off[g+1] - row_off[g]) * 32 != beta * width,
 *            is skipped (it adds nothing to Y): no read ever leaves the rows 0 .. row_off[k] - 1 that the stored form
 *            declares, also when it is read with the wrong bit_base
 * Arithmetic: codes and activations are exact; per (row, group) sum (q - z) x in fp32 (for fp16 activations on
 * the matrix cores, with 2 (q - z) formed exactly in fp16), times the scale rounded to fp32; the sums of group
 * ranges are added in a fixed order (deterministic, no atomics).
 * Uses the context's workspace for those partial sums.
 */
slim_status slim_dequant_matmul(slim_ctx* ctx, const uint32_t* packed, int64_t ldp, const uint32_t* gbits,
                                const int32_t* row_off, const double* scale, const double* zero, int n, int m,
                                int beta, int bit_base, const void* X, slim_dtype x_dtype, int t_x, int64_t ldx,
                                float* Y, int64_t ldy);

/* The same linear layer with the zero points in their packed form (App. B.2: the kernel dequantises the packed weights and
 * the packed zeros): zpacked, ldzp, zbits as slim_pack_zeros writes them; everything else as above.  The zero points are
 * unpacked into the context's workspace first (exact), so Y is bit for bit that of slim_dequant_matmul on them. */
slim_status slim_dequant_matmul_zp(slim_ctx* ctx, const uint32_t* packed, int64_t ldp, const uint32_t* gbits,
                                   const int32_t* row_off, const double* scale, const uint32_t* zpacked, int64_t ldzp,
                                   int zbits, int n, int m, int beta, int bit_base, const void* X, slim_dtype x_dtype,
                                   int t_x, int64_t ldx, float* Y, int64_t ldy);

/* ---------------------------------------------------------------------------------------------
 * n4  SliM-LLM+ on one layer (Sec. 3.4; Sec. 4; App. B; built from the list of next steps): the widths of SBA stay
 * fixed, SQC and the error compensation are left out, and every (row, group) gets a quantiser with learnable weight
 * clipping, trained with AdamW.  The paper names the borrowed method and the optimiser and no more; what is built:
 *   hi = sigmoid(gamma) max_j w_j,  lo = sigmoid(beta_p) min_j w_j,  delta = (hi - lo) / (2^b - 1),
 *   z = -round(lo / delta),  q_j = clamp(round(w_j / delta) + z, 0, 2^b - 1),  w_hat_j = delta (q_j - z)
 *   (Eq. 1 on the clipped range; every width, 1 bit included, in this affine form; a (row, group) of zeros gets delta = 1);
 *   loss L = tr((W - W_hat) G (W - W_hat)^T) / (n n_tokens), the mean squared error of the layer's outputs over the
 *   calibration tokens (Eq. 3), full batch; derivatives with the rounding taken as the identity (straight-through);
 *   gamma, beta_p start at `init` (4 in the borrowed method) and take `steps` AdamW steps (no weight decay) with
 *   step size lr and moment constants beta1, beta2, eps; the layer is then quantised with the final strengths.
 *   W      n x m, F16 / BF16 / F32, read only          G   m x m fp32 raw Gram matrix (both triangles), n_tokens its tokens
 *   bits   device, k bytes in 1..8 (from slim_sba_allocate); the call waits for them to validate them
 *   codes  n x m bytes (ld = m);  scale, zero  n x k doubles (ld = k): delta and z (integers) of every (row, group)
 *   What   optional n x m (ld = m) in what_dtype (F32 or F64), or NULL
 *   loss_curve   host, steps + 1 doubles or NULL: the loss before every step and after the last; NULL: the call does
 *          not wait for its own work
 * All arithmetic is fp64; a step costs one n x m x m product on the fp64 matrix cores and two passes over W.
 */
slim_status slim_lwc_quantize(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                              const float* G, int64_t ldg, int64_t n_tokens, const uint8_t* bits, int beta, int steps,
                              double lr, double beta1, double beta2, double eps, double init, uint8_t* codes,
                              double* scale, double* zero, void* What, slim_dtype what_dtype, double* loss_curve);

/* ---------------------------------------------------------------------------------------------
 * slim_dequant_matmul for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and launch shapes, bit for bit the same Y;
 * the partial sums of the group ranges go to a fixed buffer of SLIM_DEQUANT_NOALLOC_MAX_FLOATS floats (16 MiB) that
 * every GPU the library runs on holds from the time its code is loaded there until the process ends, instead of the
 * context's workspace.  The call allocates and frees nothing (no hipMalloc, no hipFree, no events; per-kernel timing
 * is off for its length).
 *   A layer needs (group ranges) x min(t_x, 16) x n floats, where the number of group ranges is chosen to fill the chip
 *   (about 8 x CUs / ceil(n / 128), at most k, one when that product is 1: then the buffer is not used).  If that
 *   exceeds the buffer the call returns SLIM_ERR_UNSUPPORTED and touches nothing; the error text gives the figures.
 *   All contexts on one GPU share that GPU's buffer: calls that overlap in time on one GPU (two streams) race.
 *   Nothing in it has to be zero before a call; every value read is written by the same call first.
 */
#define SLIM_DEQUANT_NOALLOC_MAX_FLOATS ((size_t)4 << 20)
slim_status slim_dequant_matmul_noalloc(slim_ctx* ctx, const uint32_t* packed, int64_t ldp, const uint32_t* gbits,
                                        const int32_t* row_off, const double* scale, const double* zero, int n,
                                        int m, int beta, int bit_base, const void* X, slim_dtype x_dtype, int t_x,
                                        int64_t ldx, float* Y, int64_t ldy);

/* ---------------------------------------------------------------------------------------------
 * Per-kernel timing with HIP events on the context's stream (measurement aid, host only).
 * While enabled, every kernel launch of the library is bracketed by an event pair.
 * An entry is named after the step of the path ("sba_output_dgemm"), followed by "@" and the kernel function
 * where the launch site chooses among several ("...@dgemm_kernel<0, 128, 128>"), followed by "#side" for a launch
 * on one of the context's internal side streams (such launches run beside the work on the context's own stream,
 * so their durations overlap it rather than add to it).
 * slim_profile_collect synchronises, folds the pending pairs into per-kernel totals and returns
 * the number of distinct kernel names; slim_profile_entry reads entry i.
 */
slim_status slim_profile_enable(slim_ctx* ctx, int on);
int slim_profile_collect(slim_ctx* ctx);
slim_status slim_profile_entry(const slim_ctx* ctx, int i, const char** name, double* total_ms, int* launches);
slim_status slim_profile_reset(slim_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* SLIM_H */
