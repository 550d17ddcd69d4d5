// a2  Damped inverse Hessian and its upper Cholesky factor (Def. 1; Alg. 1 line 2), all in fp64.
//
// Wanted: upper-triangular U with (H + lambda I)^-1 = U^T U.  Writing R = U^-1 (upper triangular) gives
// H + lambda I = R R^T, a Cholesky factorisation taken from the bottom-right corner upwards, so the
// textbook route (factor, invert, factor again) collapses to ONE factorisation and ONE triangular
// inverse, (2/3) m^3 flops instead of (4/3) m^3:
//
//   1. widen:   A = (2 / n_tokens) G + lambda I,  lambda = percdamp * mean(diag(2 / n_tokens G))
//   2. for the diagonal blocks J = last .. first (64 columns each):
//        chol_diag   A_JJ = R_JJ R_JJ^T in LDS by one workgroup, plus V_JJ = R_JJ^-1 (written into U)
//        panel       R[0:J, J] = A[0:J, J] V_JJ^T                    (fp64 MFMA GEMM)
//        update      A[0:J, 0:J] -= R[0:J, J] R[0:J, J]^T, upper tiles only   (fp64 MFMA GEMM)
//   3. triangular inverse by recursive doubling: ranges of 2^l diagonal blocks that are already inverted
//      are merged pairwise, U12 = -U11 (R12 U22); all pairs of a level form one batched GEMM launch.
//   4. hinv_diag_j = sum_i U_ij^2.
#include "slim_device.h"
#include "slim_internal.h"

namespace {

constexpr int NB = 64;          // diagonal block

// mean of the diagonal of H = s * G, then lambda; single workgroup, fixed order
__global__ __launch_bounds__(256) void damp_lambda(const float* __restrict__ G, int64_t ldg, int m, double s,
                                                   double percdamp, double* __restrict__ lam_out,
                                                   int* __restrict__ flag) {
  __shared__ double red[256];
  if (threadIdx.x == 0) *flag = 0;
  double acc = 0.0;
  for (int i = threadIdx.x; i < m; i += 256) acc += s * (double)G[(int64_t)i * ldg + i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int st = 128; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) *lam_out = percdamp * (red[0] / (double)m);
}

// A = s * G + lambda I on and above the diagonal, zero below
__global__ __launch_bounds__(256) void widen_damp(const float* __restrict__ G, int64_t ldg, int m, double s,
                                                  const double* __restrict__ lam, double* __restrict__ A,
                                                  int64_t lda) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int r = blockIdx.y;
  if (c >= m) return;
  double v = 0.0;
  if (c >= r) {
    v = s * (double)G[(int64_t)r * ldg + c];
    if (c == r) v += *lam;
  }
  A[(int64_t)r * lda + c] = v;
}

__global__ __launch_bounds__(256) void zero_matrix(double* __restrict__ A, int64_t lda, int m) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c < m) A[(int64_t)blockIdx.y * lda + c] = 0.0;
}

// 1 / x to full double precision for positive finite x: hardware estimate plus two Newton steps
__device__ __forceinline__ double fast_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = fma(fma(-x, r, 1.0), r, r);
  r = fma(fma(-x, r, 1.0), r, r);
  return r;
}

// One workgroup (16 wavefronts) factors the nbk x nbk diagonal block at A (upper triangle valid) as R R^T
// with R upper triangular, from the last column to the first, writes R back (zero below the diagonal) and
// its inverse V into Vout.  A non-positive pivot is recorded in flag[0] (1-based global column) and
// replaced by 1.
//
// A lone wavefront issues roughly one instruction every 8 cycles on this chip, so the kernel is built to
// execute few instructions per elimination step: lane = row, wavefront w owns columns w, w+16, w+32, w+48
// in four registers.  The pivot column therefore sits in ONE register of ONE wavefront and is broadcast
// with a single 64-lane LDS store; which columns still take part in a step is known statically (register
// index) or per wavefront (scalar), never per lane.  Entries below the diagonal are never read.
__global__ __launch_bounds__(1024) void chol_diag(double* __restrict__ A, int64_t lda, int nbk, double* __restrict__ Vout,
                                                  int64_t ldv, int* __restrict__ flag, int col_base) {
  constexpr int LD = NB + 1;
  __shared__ double Rs[NB * LD];       // the block (row-major), later R, later V
  __shared__ double cb[2][NB];         // broadcast column, double buffered
  __shared__ double diag[NB], rdiag[NB];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // coalesced load (lane = column), identity padding of a ragged block
  for (int r = w; r < NB; r += 16) {
    double v = (r == lane) ? 1.0 : 0.0;
    if (r < nbk && lane < nbk) v = (lane >= r) ? A[(int64_t)r * lda + lane] : 0.0;
    Rs[r * LD + lane] = v;
  }
  __syncthreads();
  double a[4], b[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    a[q] = Rs[lane * LD + w + 16 * q];
    b[q] = (lane == w + 16 * q) ? 1.0 : 0.0;
  }
  // ---- factorisation: after step j, column j holds R[:, j] * R[j][j] (scaled afterwards)
#pragma unroll
  for (int qj = 3; qj >= 0; --qj) {
    for (int wj = 15; wj >= 0; --wj) {
      const int j = 16 * qj + wj;
      double* c = cb[j & 1];
      if (w == wj) c[lane] = a[qj];
      __syncthreads();
      double piv = c[j];
      if (!(piv > 0.0)) {                                 // uniform over the workgroup, rare
        if (tid == 0 && j < nbk && flag[0] == 0) flag[0] = col_base + j + 1;
        piv = 1.0;
        if (w == wj && lane == j) a[qj] = 1.0;            // keep the sanitised pivot for the scaling pass
      }
      const double s = c[lane] * fast_rcp(piv);           // a[i][j] / pivot for this lane's row
      // columns of registers below qj are all left of j; register qj itself only in wavefronts left of wj
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (q < qj) a[q] -= s * c[w + 16 * q];
      }
      if (w < wj) a[qj] -= s * c[w + 16 * qj];
    }
  }
  // ---- scale: R[i][j] = a[i][j] / sqrt(a[j][j]); zeros below the diagonal; R goes to LDS
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (lane == w + 16 * q) {
      const double d = sqrt(a[q]);
      diag[lane] = d;
      rdiag[lane] = 1.0 / d;
    }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int cq = w + 16 * q;
    a[q] = (lane < cq) ? a[q] * rdiag[cq] : ((lane == cq) ? diag[cq] : 0.0);
    Rs[lane * LD + cq] = a[q];
  }
  __syncthreads();
  for (int r = w; r < NB; r += 16)
    if (r < nbk && lane < nbk) A[(int64_t)r * lda + lane] = Rs[r * LD + lane];
  // ---- inverse: V R = I, columns from left to right.  Column c of V is final once the columns left of it
  //      have been eliminated; it is broadcast and subtracted from the columns to its right.
#pragma unroll
  for (int qc = 0; qc < 4; ++qc) {
    for (int wc = 0; wc < 16; ++wc) {
      const int cc = 16 * qc + wc;
      double* c = cb[cc & 1];
      if (w == wc) {
        b[qc] *= rdiag[cc];
        c[lane] = b[qc];
      }
      __syncthreads();
      const double v = c[lane];
      const double* rrow = Rs + cc * LD;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (q > qc) b[q] -= v * rrow[w + 16 * q];
      }
      if (w > wc) b[qc] -= v * rrow[w + 16 * qc];
    }
  }
  __syncthreads();   // every wavefront is done reading R from LDS
#pragma unroll
  for (int q = 0; q < 4; ++q) Rs[lane * LD + w + 16 * q] = b[q];
  __syncthreads();
  for (int r = w; r < NB; r += 16)
    if (r < nbk && lane < nbk) Vout[(int64_t)r * ldv + lane] = (lane >= r) ? Rs[r * LD + lane] : 0.0;
}

// partial column sums of squares of the upper triangle of U: grid (ceil(m/64), parts); part p owns 256 rows
__global__ __launch_bounds__(256) void colsumsq_upper(const double* __restrict__ U, int64_t ldu, int m,
                                                      double* __restrict__ partial) {
  __shared__ double red[4][64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + tx;
  const int r0 = blockIdx.y * 256;
  double acc = 0.0;
  if (c < m) {
    const int r1 = min(min(m, r0 + 256), c + 1);
    for (int r = r0 + ty; r < r1; r += 4) {
      const double v = U[(int64_t)r * ldu + c];
      acc += v * v;
    }
  }
  red[ty][tx] = acc;
  __syncthreads();
  if (ty == 0 && c < m) partial[(int64_t)blockIdx.y * m + c] = ((red[0][tx] + red[1][tx]) + red[2][tx]) + red[3][tx];
}

__global__ __launch_bounds__(256) void colsum_finalize(const double* __restrict__ partial, int parts, int m,
                                                       double* __restrict__ out) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= m) return;
  double s = 0.0;
  const int pmax = min(parts, c / 256 + 1);   // parts whose rows lie above the diagonal entry of column c
  for (int p = 0; p < pmax; ++p) s += partial[(int64_t)p * m + c];
  out[c] = s;
}

}  // namespace

extern "C" slim_status slim_hessian_inverse(slim_ctx* ctx, const float* G, int64_t ldg, int m, int64_t n_tokens,
                                            double percdamp, double* U, int64_t ldu, double* hinv_diag, int* info) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, G && U && hinv_diag && info, "slim_hessian_inverse: null pointer");
  SLIM_REQUIRE(ctx, m > 0 && m % 2 == 0, "slim_hessian_inverse: m must be positive and even (got %d)", m);
  SLIM_REQUIRE(ctx, ldg >= m && ldu >= m && ldu % 2 == 0, "slim_hessian_inverse: bad leading dimension");
  SLIM_REQUIRE(ctx, n_tokens > 0, "slim_hessian_inverse: n_tokens must be positive");
  SLIM_REQUIRE(ctx, percdamp >= 0.0, "slim_hessian_inverse: percdamp must be >= 0");
  SLIM_REQUIRE(ctx, slim_aligned16(U), "slim_hessian_inverse: U must be 16-byte aligned");
  *info = 0;

  const int nblk = slim_cdiv(m, NB);
  const int64_t lda = m;
  const int parts = slim_cdiv(m, 256);
  // descriptors of the triangular inverse, built on the host
  std::vector<slim_gemm_desc> descs;
  struct Level { int first, count, maxM, maxN; };
  std::vector<Level> levels;

  const size_t bytes_A = slim_ws_round(sizeof(double) * (size_t)m * m);
  const size_t bytes_P = slim_ws_round(sizeof(double) * (size_t)m * NB * 2);   // two panels (double buffer)
  const size_t bytes_part = slim_ws_round(sizeof(double) * (size_t)parts * m);
  const size_t bytes_desc = slim_ws_round(sizeof(slim_gemm_desc) * (size_t)(2 * nblk + 8));
  slim_status st = slim_ws_reserve(ctx, 2 * bytes_A + bytes_P + bytes_part + bytes_desc + 256);
  if (st != SLIM_OK) return st;
  double* A = static_cast<double*>(slim_ws_alloc(ctx, bytes_A));
  double* T = static_cast<double*>(slim_ws_alloc(ctx, bytes_A));
  double* P = static_cast<double*>(slim_ws_alloc(ctx, bytes_P));
  double* partial = static_cast<double*>(slim_ws_alloc(ctx, bytes_part));
  slim_gemm_desc* descs_dev = static_cast<slim_gemm_desc*>(slim_ws_alloc(ctx, bytes_desc));
  double* lam = static_cast<double*>(slim_ws_alloc(ctx, 256));
  int* flag = ctx->dflags + 1;

  const double s = 2.0 / (double)n_tokens;
  SLIM_LAUNCH(ctx, "inv_lambda", damp_lambda, dim3(1), dim3(256), 0, G, ldg, m, s, percdamp, lam, flag);
  const dim3 mgrid(slim_cdiv(m, 256), m);
  SLIM_LAUNCH(ctx, "inv_widen", widen_damp, mgrid, dim3(256), 0, G, ldg, m, s, lam, A, lda);
  SLIM_LAUNCH(ctx, "inv_zero_u", zero_matrix, mgrid, dim3(256), 0, U, ldu, m);

  // ---- descriptors of the triangular inverse (pairwise merging of inverted diagonal ranges), staged first so
  //      that no host synchronisation falls between the factorisation and the inverse
  for (int64_t sz = NB; sz < m; sz *= 2) {
    Level lv{(int)descs.size(), 0, 0, 0};
    for (int64_t lo = 0; lo + sz < m; lo += 2 * sz) {
      const int64_t mid = lo + sz, hi = std::min<int64_t>(lo + 2 * sz, m);
      const int a = (int)sz, b = (int)(hi - mid);
      slim_gemm_desc d;
      // T12 = R12 * U22
      d.A = A + lo * lda + mid;
      d.lda = lda;
      d.B = U + mid * ldu + mid;
      d.ldb = ldu;
      d.C = T + lo * lda + mid;
      d.ldc = lda;
      d.C2 = nullptr;
      d.ldc2 = 0;
      d.M = a;
      d.N = b;
      d.K = b;
      d.flags = SLIM_GEMM_B_UPPER;
      d.alpha = 1.0;
      d.beta = 0.0;
      descs.push_back(d);
      lv.count += 1;
      lv.maxM = std::max(lv.maxM, a);
      lv.maxN = std::max(lv.maxN, b);
    }
    levels.push_back(lv);
  }
  const int n_first = (int)descs.size();
  // second product of every pair: U12 = -U11 * T12
  for (int i = 0; i < n_first; ++i) {
    const slim_gemm_desc& t = descs[i];
    const int64_t off = t.C - T;   // element offset of the (lo, mid) block
    const int64_t lo = off / lda, mid = off % lda;
    slim_gemm_desc d;
    d.A = U + lo * ldu + lo;
    d.lda = ldu;
    d.B = t.C;
    d.ldb = lda;
    d.C = U + lo * ldu + mid;
    d.ldc = ldu;
    d.C2 = nullptr;
    d.ldc2 = 0;
    d.M = t.M;
    d.N = t.N;
    d.K = t.M;
    d.flags = SLIM_GEMM_A_UPPER;
    d.alpha = -1.0;
    d.beta = 0.0;
    descs.push_back(d);
  }
  if (!descs.empty()) {
    if (descs.size() * sizeof(slim_gemm_desc) > (size_t)SLIM_HPIN_BYTES)
      return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_hessian_inverse: m too large for the descriptor staging buffer");
    // the staging buffer may still be read by an earlier asynchronous copy
    SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    memcpy(ctx->hpin, descs.data(), descs.size() * sizeof(slim_gemm_desc));
    SLIM_HIP_TRY(ctx, hipMemcpyAsync(descs_dev, ctx->hpin, descs.size() * sizeof(slim_gemm_desc),
                                     hipMemcpyHostToDevice, ctx->stream));
  }

  // ---- factorisation from the bottom-right corner upwards, with one block of lookahead:
  //   main stream : diag(J) -> panel(J) -> update of block column J-1 only -> diag(J-1) -> ...
  //   side stream : the bulk of the symmetric update of block J (all columns left of block J-1)
  // The bulk update therefore runs while the next diagonal block is being factored.  Events order the two
  // streams: the bulk of block J starts after panel(J); the main stream touches block column J-2 (and
  // reuses the panel buffer of block J) only after the bulk of block J has finished.
  st = slim_ensure_side(ctx);
  if (st != SLIM_OK) return st;
  hipStream_t s0 = ctx->stream, s1 = ctx->side;
  hipEvent_t ev_fork = ctx->ev[0];
  hipEvent_t ev_panel[2] = {ctx->ev[1], ctx->ev[2]};
  hipEvent_t ev_bulk[2] = {ctx->ev[3], ctx->ev[4]};
  bool bulk_issued[2] = {false, false};
  SLIM_HIP_TRY(ctx, hipEventRecord(ev_fork, s0));
  SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s1, ev_fork, 0));
  struct StreamSwap {
    slim_ctx* c;
    hipStream_t keep;
    StreamSwap(slim_ctx* cc, hipStream_t s) : c(cc), keep(cc->stream) { c->stream = s; }
    ~StreamSwap() { c->stream = keep; }
  };
  for (int blk = nblk - 1; blk >= 0; --blk) {
    const int j0 = blk * NB;
    const int nbk = std::min(NB, m - j0);
    const int pb = blk & 1;
    double* Pb = P + (size_t)pb * m * NB;
    SLIM_LAUNCH(ctx, "inv_chol_diag", chol_diag, dim3(1), dim3(1024), 0, A + (int64_t)j0 * lda + j0, lda, nbk,
                U + (int64_t)j0 * ldu + j0, ldu, flag, j0);
    if (j0 == 0) break;
    slim_gemm_desc d;
    d.A = A + j0;                       // A[0:j0, j0:j0+nbk]
    d.lda = lda;
    d.B = U + (int64_t)j0 * ldu + j0;   // V_JJ, used transposed
    d.ldb = ldu;
    d.C = Pb;
    d.ldc = NB;
    d.C2 = A + j0;                      // the panel of R replaces the panel of A
    d.ldc2 = lda;
    d.M = j0;
    d.N = nbk;
    d.K = nbk;
    d.flags = 0;
    d.alpha = 1.0;
    d.beta = 0.0;
    st = slim_dgemm(ctx, "inv_panel_dgemm", 1, d);
    if (st != SLIM_OK) return st;
    SLIM_HIP_TRY(ctx, hipEventRecord(ev_panel[pb], s0));
    // block column J-1 was last written by the bulk update of block J+1
    if (bulk_issued[pb ^ 1]) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s0, ev_bulk[pb ^ 1], 0));
    const int jn = j0 - NB;             // first column of block J-1 (j0 is a multiple of NB here)
    d.A = Pb;
    d.lda = NB;
    d.B = Pb + (size_t)jn * NB;         // rows of the panel that belong to block J-1
    d.ldb = NB;
    d.C = A + jn;
    d.ldc = lda;
    d.C2 = nullptr;
    d.ldc2 = 0;
    d.M = j0;
    d.N = NB;
    d.K = nbk;
    d.flags = 0;
    d.alpha = -1.0;
    d.beta = 1.0;
    st = slim_dgemm(ctx, "inv_syrk_next_dgemm", 1, d);
    if (st != SLIM_OK) return st;
    if (jn > 0) {
      StreamSwap swap(ctx, s1);
      SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s1, ev_panel[pb], 0));
      d.B = Pb;
      d.C = A;
      d.M = jn;
      d.N = jn;
      d.flags = SLIM_GEMM_UPPER_ONLY;
      st = slim_dgemm(ctx, "inv_syrk_dgemm", 1, d);
      if (st != SLIM_OK) return st;
      SLIM_HIP_TRY(ctx, hipEventRecord(ev_bulk[pb], s1));
      bulk_issued[pb] = true;
    }
  }
  for (int i = 0; i < 2; ++i)
    if (bulk_issued[i]) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s0, ev_bulk[i], 0));

  // ---- triangular inverse U = R^-1: two batched GEMM launches per level
  if (!descs.empty()) {
    for (const Level& lv : levels) {
      if (lv.count == 0) continue;
      st = slim_dgemm_batched(ctx, "inv_trtri_dgemm", 0, descs_dev + lv.first, lv.count, lv.maxM, lv.maxN);
      if (st != SLIM_OK) return st;
      st = slim_dgemm_batched(ctx, "inv_trtri_dgemm", 0, descs_dev + n_first + lv.first, lv.count, lv.maxM, lv.maxN);
      if (st != SLIM_OK) return st;
    }
  }

  SLIM_LAUNCH(ctx, "inv_diag_colsumsq", colsumsq_upper, dim3(slim_cdiv(m, 64), parts), dim3(256), 0, U, ldu, m, partial);
  SLIM_LAUNCH(ctx, "inv_diag_finalize", colsum_finalize, dim3(slim_cdiv(m, 256)), dim3(256), 0, partial, parts, m, hinv_diag);

  int* host = reinterpret_cast<int*>(ctx->hpin);
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(host, flag, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  *info = host[0];
  if (host[0] != 0)
    return slim_fail(ctx, SLIM_ERR_NOT_PD, "slim_hessian_inverse: H + lambda I is not positive definite (pivot at column %d)", host[0]);
  return SLIM_OK;
}
