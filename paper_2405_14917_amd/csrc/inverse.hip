// a2  Damped inverse Hessian and its upper Cholesky factor (Def. 1; Alg. 1 line 2), all in fp64.
//
// Wanted: upper-triangular U with (H + lambda I)^-1 = U^T U.  Writing R = U^-1 (upper triangular) gives
// H + lambda I = R R^T, a Cholesky factorisation taken from the bottom-right corner upwards, so the
// textbook route (factor, invert, factor again) collapses to ONE factorisation and ONE triangular
// inverse, (2/3) m^3 flops instead of (4/3) m^3:
//
//   1. widen:   A = (2 / n_tokens) G + lambda I,  lambda = percdamp * mean(diag(2 / n_tokens G))
//   2. for the diagonal blocks J = last .. first (64 columns each; eight of them form a group):
//        chol_step   one workgroup: applies the last pending rank-64 update to A_JJ itself, factors
//                    A_JJ = R_JJ R_JJ^T in LDS and inverts R_JJ (V_JJ, written into U)
//        panel       R[0:J, J] = A[0:J, J] V_JJ^T                            (fp64 MFMA GEMM)
//        update      rank-64 update of the columns between the start of block J-1's group and block J
//        group update  rank-512 updates of everything further left, once per group
//      The factorisation of the diagonal blocks and the GEMMs form two chains on two streams that only
//      meet two steps apart, see the schedule at the call site.
//   3. triangular inverse U = R^-1 group by group on a further stream, beside the factorisation: inside a group
//      by recursive doubling (ranges of 2^l inverted diagonal blocks merged pairwise, U12 = -U11 (R12 U22)), the
//      rows right of the group from T = R[g, S] U[S, S], which is kept up to date for all rows above by one
//      rank-512 product per finished group (see the schedule at the call site).
//   4. hinv_diag_j = sum_i U_ij^2.
#include "slim_device.h"
#include "slim_internal.h"

namespace {

using slimdev::read_lane_f64;

constexpr int NB = 64;          // diagonal block
// Diagonal blocks per group.  With 8 the far updates have rank 512 (64 flops per byte of A they move, against 32 with
// 4) and there are half as many of them; the windows of the chain get wider.  Inverse alone at m = 11008: 21.7 against
// 22.2 ms; whole pass: 0.5 ms less on the 4096 x 11008 and 28672 x 8192 layers, 0.2 ms less on 4096 x 4096.
constexpr int GRP = 8;

// mean of the diagonal of H = s * G, then lambda; single workgroup, fixed order
__global__ __launch_bounds__(1024) void damp_lambda(const float* __restrict__ G, int64_t ldg, int m, double s,
                                                    double percdamp, double* __restrict__ lam_out,
                                                    int* __restrict__ flag) {
  __shared__ double red[1024];
  if (threadIdx.x == 0) *flag = 0;
  double acc = 0.0;
  for (int i = threadIdx.x; i < m; i += 1024) acc += s * (double)G[(int64_t)i * ldg + i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int st = 512; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) *lam_out = percdamp * (red[0] / (double)m);
}

// A = s * G + lambda I on and above the diagonal; U = 0 below it.  V consecutive columns per thread.
// What lies below the diagonal of A is never read as a value that matters (the updates that sweep over it only
// add to it), and every element of U on or above the diagonal is written later (the inverted diagonal blocks,
// then the merged off-diagonal ones), so pieces entirely on one side are written to one matrix only.
template <int V>
__global__ __launch_bounds__(256) void widen_damp(const float* __restrict__ G, int64_t ldg, int m, double s,
                                                  const double* __restrict__ lam, double* __restrict__ A,
                                                  int64_t lda, double* __restrict__ U, int64_t ldu) {
  constexpr int ROWS = 8;                      // rows per thread: the loads of all of them are issued first
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * V;
  const int r0 = blockIdx.y * ROWS;
  if (c0 >= m) return;
  float g[ROWS][V];
#pragma unroll
  for (int q = 0; q < ROWS; ++q) {
    const int r = r0 + q;
#pragma unroll
    for (int v = 0; v < V; ++v) g[q][v] = 0.0f;
    if (r < m && c0 + V - 1 >= r) {            // something of this piece lies on or above the diagonal
      const float* src = G + (int64_t)r * ldg + c0;
      if (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(src);
        g[q][0] = t.x, g[q][1] = t.y, g[q][2] = t.z, g[q][3] = t.w;
      } else if (V == 2) {
        const float2 t = *reinterpret_cast<const float2*>(src);
        g[q][0] = t.x, g[q][1] = t.y;
      } else {
        g[q][0] = src[0];
      }
    }
  }
  const double lambda = *lam;
#pragma unroll
  for (int q = 0; q < ROWS; ++q) {
    const int r = r0 + q;
    if (r >= m) break;
    double a[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const int c = c0 + v;
      a[v] = c >= r ? s * (double)g[q][v] : 0.0;
      if (c == r) a[v] += lambda;
    }
    double* da = A + (int64_t)r * lda + c0;
    double* du = U + (int64_t)r * ldu + c0;
    const bool upper = c0 + V - 1 >= r;        // has an element on or above the diagonal
    const bool lower = c0 < r;                 // has an element below it
    if (V == 1) {
      if (upper) da[0] = a[0];
      if (lower) du[0] = 0.0;
    } else {
#pragma unroll
      for (int v = 0; v < V; v += 2) {
        if (upper) *reinterpret_cast<double2*>(da + v) = make_double2(a[v], a[v + 1]);
        if (lower) *reinterpret_cast<double2*>(du + v) = make_double2(0.0, 0.0);
      }
    }
  }
}

// 1 / x to full double precision for positive finite x: hardware estimate plus two Newton steps
__device__ __forceinline__ double fast_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = fma(fma(-x, r, 1.0), r, r);
  r = fma(fma(-x, r, 1.0), r, r);
  return r;
}

typedef double double4v __attribute__((ext_vector_type(4)));

struct CholArgs {
  const double* A;       // A[j0][j0]: the diagonal block (upper triangle valid)
  int64_t lda;
  int nbk;               // width of this block (64, less for a ragged last block)
  int nprev;             // width of block J+1 whose rank-64 update is still pending on this block (0: none)
  const double* Vprev;   // V of block J+1 (in U)
  double* Vout;          // V of this block (in U)
  int64_t ldv;
  int* flag;
  int col_base;
};


// One workgroup (16 wavefronts) per diagonal block:
//   prologue   (nprev > 0)  Rn = A[J, J+1] V_{J+1}^T and A_JJ -= Rn Rn^T on the matrix cores: the update
//              with the panel of block J+1 restricted to this block, so that this kernel does not have to
//              wait for the GEMMs of block J+1
//   factor     A_JJ = R R^T with R upper triangular, from the last column to the first, and in its shadow
//   invert     V = R^-1, written to Vout (zeros below the diagonal)
// A non-positive pivot is recorded in flag[0] (1-based global column); the outputs are then meaningless.
//
// With a_j the column of pivot j at the time it is eliminated, p_j its diagonal entry and s_j = a_j / p_j,
// R = [s_j] diag(sqrt p_j), and R^-1 = diag(1 / sqrt p_j) E where E results from the identity by the row
// operations row_i -= s_j[i] row_j (i < j) in the order of the elimination.  E has columns, a column c is only
// touched by pivots j <= c, i.e. once the column c of A is finished: the wavefronts that are done factoring
// carry the inverse, the others the factorisation, and no separate inversion pass is needed.
//
// A lone wavefront issues an instruction every ~8 cycles and a dependent fp64 one every ~32, and an LDS
// write -> barrier -> read costs ~200 cycles, so the elimination is blocked by four columns: lane = row,
// wavefront w owns columns 4w .. 4w+3 of A and of E in registers.  The owner of the current four columns reads
// their 4 x 4 diagonal block with lane reads, runs its elimination on wavefront-uniform values (the serial
// chain: four reciprocals and the pivot updates between them), finishes the four columns, and publishes them
// and the s_j through LDS once; the other wavefronts apply a rank-4 update to their columns of A or E:
// 16 barriers instead of 128.  Entries of A below the diagonal are never read as values that matter.
__global__ __launch_bounds__(1024) void chol_step(CholArgs g) {
  constexpr int LD = NB + 1;
  extern __shared__ __align__(16) double sm[];
  double* Rs = sm;                 // [64][LD] staging: the block, then A[J, J+1], then Rn; later 1 / sqrt(pivot)
  double* Xs = sm + NB * LD;       // [64][LD] staging: V_{J+1}, then Rn Rn^T; then the broadcast buffers; then V
  double* cbA = Xs;                // [2][4][64] published columns
  double* cbS = Xs + 512;          // [2][4][64] the same divided by their pivots, zero at and below the pivot
  double* cbE = Xs + 1024;         // [2][4][64] combinations of the latter that drive the inverse
  double* rsq = Rs;                // [64]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nbk = g.nbk, np = g.nprev;
  const int prior_flag = g.flag[0];
  // every global load is issued up front, coalesced (lane = column): the block (identity padding of a ragged
  // one), and for the prologue A[J, J+1] and V_{J+1} (zero padding)
  double ld_d[4], ld_a[4], ld_v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = w + 16 * i;
    ld_d[i] = (r == lane) ? 1.0 : 0.0;
    if (r < nbk && lane < nbk) ld_d[i] = (lane >= r) ? g.A[(int64_t)r * g.lda + lane] : 0.0;
    ld_a[i] = 0.0;
    ld_v[i] = 0.0;
    if (np > 0) {
      if (lane < np) ld_a[i] = g.A[(int64_t)r * g.lda + NB + lane];
      if (r < np && lane < np && lane >= r) ld_v[i] = g.Vprev[(int64_t)r * g.ldv + lane];
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) Rs[(w + 16 * i) * LD + lane] = ld_d[i];
  __syncthreads();
  double a[4], e[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    a[q] = Rs[lane * LD + 4 * w + q];
    e[q] = (lane == 4 * w + q) ? 1.0 : 0.0;
  }
  if (np > 0) {
    // Rn = A[J, J+1] V^T, then A_JJ -= Rn Rn^T, as 16 x 16 MFMA tiles.  Operand lane (l16, lk) feeds row / column
    // l16 at k = 16 lk + s in step s (any assignment of k works as long as both operands share it); result
    // register v is row 4 v + lk, column l16 of the tile.
    const int l16 = lane & 15, lk = lane >> 4;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      Rs[(w + 16 * i) * LD + lane] = ld_a[i];
      Xs[(w + 16 * i) * LD + lane] = ld_v[i];
    }
    __syncthreads();
    {
      // tile (ti, tj); V[c][k] = 0 for k < c, so tile column tj needs k >= 16 tj only: lane groups lk >= tj.
      // Wavefronts that share a SIMD (w mod 4) get different tj, which balances the work.
      const int ti = w & 3, tj = w >> 2;
      double4v acc = {0.0, 0.0, 0.0, 0.0};
      const double* ap = Rs + (16 * ti + l16) * LD + 16 * lk;
      const double* bp = Xs + (16 * tj + l16) * LD + 16 * lk;
#pragma unroll
      for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[s], bp[s], acc, 0, 0, 0);
      __syncthreads();
#pragma unroll
      for (int v = 0; v < 4; ++v) Rs[(16 * ti + 4 * v + lk) * LD + 16 * tj + l16] = acc[v];
    }
    __syncthreads();
    if (w < 10) {
      // the ten tiles on and above the diagonal, dealt round the SIMDs
      const int ti = (w < 4) ? 0 : ((w < 7) ? 1 : ((w < 9) ? 2 : 3));
      const int tj = (w < 4) ? w : ((w < 7) ? w - 3 : ((w < 9) ? w - 5 : 3));
      double4v acc = {0.0, 0.0, 0.0, 0.0};
      const double* ap = Rs + (16 * ti + l16) * LD + 16 * lk;
      const double* bp = Rs + (16 * tj + l16) * LD + 16 * lk;
#pragma unroll
      for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(ap[s], bp[s], acc, 0, 0, 0);
#pragma unroll
      for (int v = 0; v < 4; ++v) Xs[(16 * ti + 4 * v + lk) * LD + 16 * tj + l16] = acc[v];
    }
    __syncthreads();
    // below the diagonal Xs still holds entries of V: finite, and never used as values that matter
#pragma unroll
    for (int q = 0; q < 4; ++q) a[q] -= Xs[lane * LD + 4 * w + q];
  }
  __syncthreads();   // Rs and Xs are free from here on
  int bad = 0;       // owner only: a non-positive pivot in this lane's column

  // E lags one step behind: in step wj the wavefronts right of the owner apply the row operations of the
  // pivots of step wj+1, whose owner prepared them after its barrier, off the critical path.
  auto e_update = [&](const double* bE, int jp) {
    double sp[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) sp[r] = bE[r * 64 + lane];
#pragma unroll
    for (int q2 = 0; q2 < 4; ++q2) {
      const double x0 = read_lane_f64(e[q2], jp), x1 = read_lane_f64(e[q2], jp + 1);
      const double x2 = read_lane_f64(e[q2], jp + 2), x3 = read_lane_f64(e[q2], jp + 3);
      e[q2] = fma(-sp[0], x0, fma(-sp[1], x1, fma(-sp[2], x2, fma(-sp[3], x3, e[q2]))));
    }
  };
  for (int wj = 15; wj >= 0; --wj) {
    double* bA = cbA + (wj & 1) * 256;
    double* bS = cbS + (wj & 1) * 256;
    const int jb = 4 * wj;
    double pj = 1.0, sv0 = 0.0, sv1 = 0.0, sv2 = 0.0, sv3 = 0.0;
    if (w == wj) {
      // the 4 x 4 diagonal block of the owner's columns: D_rc = a[c] at row jb + r  (r <= c), uniform values
      const double D33 = read_lane_f64(a[3], jb + 3), D23 = read_lane_f64(a[3], jb + 2);
      const double D13 = read_lane_f64(a[3], jb + 1), D03 = read_lane_f64(a[3], jb + 0);
      const double D22 = read_lane_f64(a[2], jb + 2), D12 = read_lane_f64(a[2], jb + 1);
      const double D02 = read_lane_f64(a[2], jb + 0), D11 = read_lane_f64(a[1], jb + 1);
      const double D01 = read_lane_f64(a[1], jb + 0), D00 = read_lane_f64(a[0], jb + 0);
      // elimination of the block on uniform values; the chain is r3 -> p2 -> r2 -> p1 -> r1 -> p0 -> r0
      const double r3 = fast_rcp(D33);
      const double p2 = fma(-(D23 * D23), r3, D22);
      const double E12 = fma(-(D13 * D23), r3, D12);       // entries after pivot 3
      const double E02 = fma(-(D03 * D23), r3, D02);
      const double E11 = fma(-(D13 * D13), r3, D11);
      const double E01 = fma(-(D03 * D13), r3, D01);
      const double E00 = fma(-(D03 * D03), r3, D00);
      const double r2 = fast_rcp(p2);
      const double p1 = fma(-(E12 * E12), r2, E11);
      const double F01 = fma(-(E02 * E12), r2, E01);       // entries after pivot 2
      const double F00 = fma(-(E02 * E02), r2, E00);
      const double r1 = fast_rcp(p1);
      const double p0 = fma(-(F01 * F01), r1, F00);
      const double r0 = fast_rcp(p0);
      // the four columns as they stand when they are eliminated, and s_j = a_j / p_j
      const double s3 = a[3] * r3;
      a[2] = fma(-s3, D23, a[2]);
      const double s2 = a[2] * r2;
      a[1] = fma(-s2, E12, fma(-s3, D13, a[1]));
      const double s1 = a[1] * r1;
      a[0] = fma(-s1, F01, fma(-s2, E02, fma(-s3, D03, a[0])));
      const double s0 = a[0] * r0;
      // rows at and below the pivot take no part in the row operations
      sv0 = (lane < jb + 0) ? s0 : 0.0;
      sv1 = (lane < jb + 1) ? s1 : 0.0;
      sv2 = (lane < jb + 2) ? s2 : 0.0;
      sv3 = (lane < jb + 3) ? s3 : 0.0;
      bA[0 * 64 + lane] = a[0];
      bA[1 * 64 + lane] = a[1];
      bA[2 * 64 + lane] = a[2];
      bA[3 * 64 + lane] = a[3];
      bS[0 * 64 + lane] = sv0;
      bS[1 * 64 + lane] = sv1;
      bS[2 * 64 + lane] = sv2;
      bS[3 * 64 + lane] = sv3;
      pj = (lane == jb + 3) ? D33 : ((lane == jb + 2) ? p2 : ((lane == jb + 1) ? p1 : p0));
    }
    __syncthreads();
    if (w < wj) {
      // factorisation: rank-4 update of this wavefront's columns of A
      double s4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) s4[q] = bS[q * 64 + lane];
#pragma unroll
      for (int q = 3; q >= 0; --q) {
        const double2 c01 = *reinterpret_cast<const double2*>(&bA[q * 64 + 4 * w]);
        const double2 c23 = *reinterpret_cast<const double2*>(&bA[q * 64 + 4 * w + 2]);
        a[0] = fma(-s4[q], c01.x, a[0]);
        a[1] = fma(-s4[q], c01.y, a[1]);
        a[2] = fma(-s4[q], c23.x, a[2]);
        a[3] = fma(-s4[q], c23.y, a[3]);
      }
    } else if (w == wj) {
      // Off the chain.  With x_r the entries of a column of E in the pivot rows before this block's row
      // operations, the rows the four operations use are
      //   y3 = x3, y2 = x2 - t32 y3, y1 = x1 - t31 y3 - t21 y2, y0 = x0 - t30 y3 - t20 y2 - t10 y1,  t_qr = s_q[jb+r],
      // and every row i loses sum_q s_q[i] y_q = sum_r s'_r[i] x_r; the s'_r are published for the next step.
      const double t32 = read_lane_f64(sv3, jb + 2), t31 = read_lane_f64(sv3, jb + 1), t30 = read_lane_f64(sv3, jb);
      const double t21 = read_lane_f64(sv2, jb + 1), t20 = read_lane_f64(sv2, jb), t10 = read_lane_f64(sv1, jb);
      const double L13 = fma(t21, t32, -t31);
      const double L02 = fma(t10, t21, -t20);
      const double L03 = fma(-t10, L13, fma(t20, t32, -t30));
      double* bE = cbE + (wj & 1) * 256;
      bE[0 * 64 + lane] = sv0;
      bE[1 * 64 + lane] = fma(-t10, sv0, sv1);
      bE[2 * 64 + lane] = fma(L02, sv0, fma(-t21, sv1, sv2));
      bE[3 * 64 + lane] = fma(L03, sv0, fma(L13, sv1, fma(-t32, sv2, sv3)));
      if (lane >= jb && lane < jb + 4) {
        rsq[lane] = 1.0 / sqrt(pj);                        // for the final scaling
        if (!(pj > 0.0) && lane < nbk) bad = 1;
      }
    } else {
      e_update(cbE + ((wj + 1) & 1) * 256, jb + 4);
    }
  }
  __syncthreads();
  e_update(cbE, 0);   // the pivots of the last step (columns 0 .. 3) act on every column
  // the first failure in elimination order is kept: the highest column of the first block that fails
  if (bad && prior_flag == 0) atomicMax(g.flag, g.col_base + lane + 1);
  __syncthreads();   // every wavefront is done with the broadcast buffers, which V now overwrites
  const double rs = rsq[lane];
#pragma unroll
  for (int q = 0; q < 4; ++q) Xs[lane * LD + 4 * w + q] = e[q] * rs;
  __syncthreads();
  for (int r = w; r < NB; r += 16)
    if (r < nbk && lane < nbk) g.Vout[(int64_t)r * g.ldv + lane] = (lane >= r) ? Xs[r * LD + lane] : 0.0;
}

constexpr size_t CHOL_LDS = sizeof(double) * 2 * NB * (NB + 1);

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

size_t slim_ws_need_inverse(int m) {
  const int nblk = slim_cdiv(m, NB), parts = slim_cdiv(m, 256);
  return 2 * slim_ws_round(sizeof(double) * (size_t)m * m) + slim_ws_round(sizeof(double) * (size_t)parts * m) +
         slim_ws_round(sizeof(slim_gemm_desc) * (size_t)(2 * nblk + 8)) + 256;
}

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

  // A: the matrix being factored (upper triangle), later the scratch of the triangular inverse.
  // R: the factor, panel by panel (only the blocks above the diagonal are ever written or read).
  const size_t bytes_A = slim_ws_round(sizeof(double) * (size_t)m * m);
  const size_t bytes_part = slim_ws_round(sizeof(double) * (size_t)parts * m);
  const size_t bytes_desc = slim_ws_round(sizeof(slim_gemm_desc) * (size_t)(2 * nblk + 8));
  slim_status st = slim_ws_reserve(ctx, slim_ws_need_inverse(m));
  if (st != SLIM_OK) return st;
  double* A = static_cast<double*>(slim_ws_alloc(ctx, bytes_A));
  double* R = static_cast<double*>(slim_ws_alloc(ctx, bytes_A));
  double* partial = static_cast<double*>(slim_ws_alloc(ctx, bytes_part));
  slim_gemm_desc* descs_dev = static_cast<slim_gemm_desc*>(slim_ws_alloc(ctx, bytes_desc));
  double* lam = static_cast<double*>(slim_ws_alloc(ctx, 256));
  int* flag = ctx->dflags + 1;

  const double s = 2.0 / (double)n_tokens;
  SLIM_LAUNCH(ctx, "inv_lambda", damp_lambda, dim3(1), dim3(1024), 0, G, ldg, m, s, percdamp, lam, flag);
  // one pass writes A (widened, damped) and clears U; 4 / 2 / 1 columns per thread as alignment allows
  const bool g16 = (reinterpret_cast<uintptr_t>(G) & 15u) == 0, g8 = (reinterpret_cast<uintptr_t>(G) & 7u) == 0;
  if (m % 4 == 0 && ldg % 4 == 0 && ldu % 4 == 0 && g16)
    SLIM_LAUNCH(ctx, "inv_widen", widen_damp<4>, dim3(slim_cdiv(m, 1024), slim_cdiv(m, 8)), dim3(256), 0, G, ldg, m, s, lam, A, lda, U, ldu);
  else if (ldg % 2 == 0 && g8)
    SLIM_LAUNCH(ctx, "inv_widen", widen_damp<2>, dim3(slim_cdiv(m, 512), slim_cdiv(m, 8)), dim3(256), 0, G, ldg, m, s, lam, A, lda, U, ldu);
  else
    SLIM_LAUNCH(ctx, "inv_widen", widen_damp<1>, dim3(slim_cdiv(m, 256), slim_cdiv(m, 8)), dim3(256), 0, G, ldg, m, s, lam, A, lda, U, ldu);

  // ---- descriptors of the triangular inverse inside the groups (pairwise merging of inverted diagonal ranges),
  //      staged first so that no host synchronisation falls inside the factorisation
  const int ngrp = slim_cdiv(nblk, GRP);
  std::vector<std::vector<Level>> glevels(ngrp);
  for (int Gi = 0; Gi < ngrp; ++Gi) {
    const int64_t g0 = (int64_t)Gi * GRP * NB, g1 = std::min<int64_t>(m, g0 + GRP * NB);
    for (int64_t sz = NB; sz < g1 - g0; sz *= 2) {
      Level lv{(int)descs.size(), 0, 0, 0};
      for (int64_t lo = g0; lo + sz < g1; lo += 2 * sz) {
        const int64_t mid = lo + sz, hi = std::min<int64_t>(lo + 2 * sz, g1);
        const int a = (int)sz, b = (int)(hi - mid);
        slim_gemm_desc d;
        // T12 = R12 * U22 (into the scratch, at the position of the block)
        d.A = R + lo * lda + mid;
        d.lda = lda;
        d.B = U + mid * ldu + mid;
        d.ldb = ldu;
        d.C = A + lo * lda + mid;
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
      glevels[Gi].push_back(lv);
    }
  }
  const int n_first = (int)descs.size();
  // second product of every pair: U12 = -U11 * T12
  for (int i = 0; i < n_first; ++i) {
    const slim_gemm_desc& t = descs[i];
    const int64_t off = t.C - A;   // element offset of the (lo, mid) block
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
    // The staging buffer may still be read by the copy of an earlier call that ended on an error; every other use
    // of it has been waited for.  No wait for the stream itself: the launches of the factorisation below are
    // enqueued while earlier work (the Gram matrix) still runs, so its chain of small kernels finds them ready.
    st = slim_ensure_side(ctx);
    if (st != SLIM_OK) return st;
    if (ctx->staging_copy_pending) SLIM_HIP_TRY(ctx, hipEventSynchronize(ctx->ev[13]));
    memcpy(ctx->hpin, descs.data(), descs.size() * sizeof(slim_gemm_desc));
    SLIM_HIP_TRY(ctx, hipMemcpyAsync(descs_dev, ctx->hpin, descs.size() * sizeof(slim_gemm_desc),
                                     hipMemcpyHostToDevice, ctx->stream));
    SLIM_HIP_TRY(ctx, hipEventRecord(ctx->ev[13], ctx->stream));
    ctx->staging_copy_pending = true;
  }

  // ---- factorisation from the bottom-right corner upwards.  Blocks of 64 columns, groups of GRP blocks;
  //      "the window of block K" = the columns from the start of the group of block K-1 up to block K.
  //   s0 (caller's stream)  step(J): the diagonal-block kernel; it applies the update with panel J+1 to A_JJ
  //                         itself, so it depends on step(J+1) and on the GEMMs of block J+2 only
  //   s1  gemm(K):          panel R[0:K, K] = A[0:K, K] V_KK^T
  //                         A[rows above block K-1, window of K] -= R[.., K] R[window, K]^T        (rank 64)
  //                         and, when K is the second block of its group G (all other panels of G are done):
  //                         A[0:G, columns of group G-1] -= the panels of G except the first block's
  //   s2  far(G):           A[left of group G-1]^2 -= all panels of G, upper tiles only            (rank 512)
  // Every element of A thus receives each panel's contribution exactly once: from far() if it lies two or more
  // groups to the left, from the group update if one group to the left (the first block's panel comes through
  // that block's window), from a window update inside the group, and from the diagonal kernel for the
  // neighbouring diagonal block.  gemm(K) runs while step(K-1) runs; step(K-2) waits for it.
  st = slim_ensure_side(ctx);
  if (st != SLIM_OK) return st;
  {
    static bool done = false;
    if (!done) {
      SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(chol_step),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)CHOL_LDS));
      done = true;
    }
  }
  hipStream_t s0 = ctx->stream, s1 = ctx->side, s2 = ctx->side2, s3 = ctx->side3;
  hipEvent_t ev_fork = ctx->ev[0];
  hipEvent_t* ev_step = &ctx->ev[1];   // ring of 4
  hipEvent_t* ev_gemm = &ctx->ev[5];   // ring of 4
  hipEvent_t* ev_far = &ctx->ev[9];    // ring of 2
  SLIM_HIP_TRY(ctx, hipEventRecord(ev_fork, s0));
  SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s1, ev_fork, 0));
  SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s2, ev_fork, 0));
  SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s3, ev_fork, 0));
  struct StreamSwap {
    slim_ctx* c;
    hipStream_t keep;
    StreamSwap(slim_ctx* cc, hipStream_t s) : c(cc), keep(cc->stream) {
      c->stream = s;
      c->on_side = true;
    }
    ~StreamSwap() {
      c->stream = keep;
      c->on_side = false;
    }
  };
  struct AttachGuard {  // no event stays offered to a later call's launch when this one returns early
    slim_ctx* c;
    ~AttachGuard() { c->attach_event = nullptr; }
  } attach_guard{ctx};
  // ---- s3: the triangular inverse U = R^-1, group by group behind the factorisation.  With S the columns right of
  //      group g, U[g, S] = -U[g, g] T[g, S] where T[g, S] = R[g, S] U[S, S] = sum over the groups h in S of
  //      R[g, h] U[h, S]: the term of group h exists as soon as the rows U[h, :] do, for all rows above h at once
  //      (a rank-512 product with a large result, like the far updates of the factorisation), so that the whole
  //      inverse runs beside the factorisation, whose second half is a chain of small kernels on a nearly idle chip,
  //      and only the last group's share is left when the last diagonal block is done.  Per group, in this order:
  //        inside   U[g, g] by recursive doubling: ranges of 2^l inverted diagonal blocks are merged pairwise,
  //                 U12 = -U11 (R12 U22); all pairs of a level form one batched launch
  //        rows     U[g, S] = -U[g, g] T[g, S]
  //        terms    T[0:g0, g0:m] (+)= R[0:g0, g] U[g, g0:m]   (first term of the columns of g itself, added to the
  //                 columns right of it)
  //      T lives in A right of the group, where the panels' inputs lay: the last reader of those columns of A is the
  //      diagonal kernel of the block left of the group (its pending rank-64 update), which the caller waits for.
  auto group_inverse = [&](int Gi) -> slim_status {
    StreamSwap swap(ctx, s3);
    const int64_t g0 = (int64_t)Gi * GRP * NB, g1 = std::min<int64_t>(m, g0 + GRP * NB);
    const int gw = (int)(g1 - g0);
    slim_status rs;
    for (const Level& lv : glevels[Gi]) {
      if (lv.count == 0) continue;
      rs = slim_dgemm_batched(ctx, "inv_trtri_dgemm", 0, descs_dev + lv.first, lv.count, lv.maxM, lv.maxN);
      if (rs != SLIM_OK) return rs;
      rs = slim_dgemm_batched(ctx, "inv_trtri_dgemm", 0, descs_dev + n_first + lv.first, lv.count, lv.maxM, lv.maxN);
      if (rs != SLIM_OK) return rs;
    }
    slim_gemm_desc d;
    d.C2 = nullptr;
    d.ldc2 = 0;
    if (g1 < m) {
      d.A = U + g0 * ldu + g0;
      d.lda = ldu;
      d.B = A + g0 * lda + g1;
      d.ldb = lda;
      d.C = U + g0 * ldu + g1;
      d.ldc = ldu;
      d.M = gw;
      d.N = (int)(m - g1);
      d.K = gw;
      d.flags = SLIM_GEMM_A_UPPER;
      d.alpha = -1.0;
      d.beta = 0.0;
      rs = slim_dgemm(ctx, "inv_trtri_rows_dgemm", 0, d);
      if (rs != SLIM_OK) return rs;
    }
    if (g0 > 0) {
      d.A = R + g0;
      d.lda = lda;
      d.B = U + g0 * ldu + g0;
      d.ldb = ldu;
      d.C = A + g0;
      d.ldc = lda;
      d.M = (int)g0;
      d.N = gw;
      d.K = gw;
      d.flags = SLIM_GEMM_B_UPPER;
      d.alpha = 1.0;
      d.beta = 0.0;
      rs = slim_dgemm(ctx, "inv_trtri_terms_dgemm", 0, d);
      if (rs != SLIM_OK) return rs;
      if (g1 < m) {
        d.B = U + g0 * ldu + g1;
        d.C = A + g1;
        d.N = (int)(m - g1);
        d.flags = 0;
        d.beta = 1.0;
        rs = slim_dgemm(ctx, "inv_trtri_terms_dgemm", 0, d);
        if (rs != SLIM_OK) return rs;
      }
    }
    return SLIM_OK;
  };
  bool far_issued = false;
  int last_far_slot = 0;
  for (int J = nblk - 1; J >= 0; --J) {
    const int j0 = J * NB;
    const int nbk = std::min(NB, m - j0);
    // ---- s0: diagonal block
    if (J + 2 <= nblk - 1) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s0, ev_gemm[(J + 2) & 3], 0));
    CholArgs ca;
    ca.A = A + (int64_t)j0 * lda + j0;
    ca.lda = lda;
    ca.nbk = nbk;
    ca.nprev = (J < nblk - 1) ? std::min(NB, m - (j0 + NB)) : 0;
    ca.Vprev = U + (int64_t)(j0 + NB) * ldu + (j0 + NB);
    ca.Vout = U + (int64_t)j0 * ldu + j0;
    ca.ldv = ldu;
    ca.flag = flag;
    ca.col_base = j0;
    // The event that the GEMMs of this block wait for rides on the kernel's own completion signal (a separate record
    // is one more packet for the command processor between two diagonal steps, whose chain is what the
    // factorisation takes).
    if (J > 0) ctx->attach_event = ev_step[J & 3];
    SLIM_LAUNCH(ctx, "inv_chol_diag", chol_step, dim3(1), dim3(1024), CHOL_LDS, ca);
    if (J == 0) break;
    SLIM_HIP_TRY(ctx, slim_attach_flush(ctx));
    // ---- s3: the group to the right is factored, its panels are complete (GEMMs of its first block), and with this
    //      diagonal step the last reader of A right of this block is under way
    if ((J + 1) % GRP == 0 && J + 1 < nblk) {
      SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s3, ev_gemm[(J + 1) & 3], 0));
      SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s3, ev_step[J & 3], 0));
      st = group_inverse((J + 1) / GRP);
      if (st != SLIM_OK) return st;
    }

    // ---- s1: GEMMs of block J
    const int G = J / GRP;                          // group of block J
    const int g0 = G * GRP * NB;                    // first column of the group
    const int g1 = std::min(m, g0 + GRP * NB);      // one past its last column
    const int wstart = ((J - 1) / GRP) * GRP * NB;  // window: from the start of the group of block J-1 ...
    const int jn = j0 - NB;                         // ... to block J; rows above block J-1 take part
    {
      StreamSwap swap(ctx, s1);
      SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s1, ev_step[J & 3], 0));
      slim_gemm_desc d;
      d.A = A + j0;                       // A[0:j0, j0:j0+nbk]
      d.lda = lda;
      d.B = U + (int64_t)j0 * ldu + j0;   // V_JJ, used transposed
      d.ldb = ldu;
      d.C = R + j0;
      d.ldc = lda;
      d.C2 = nullptr;
      d.ldc2 = 0;
      d.M = j0;
      d.N = nbk;
      d.K = nbk;
      d.flags = SLIM_GEMM_CHAIN;
      d.alpha = 1.0;
      d.beta = 0.0;
      // the stage's event goes with its last launch
      const bool has_window = jn > 0;
      const bool has_group = J == G * GRP + 1 && g0 > 0;
      if (!has_window && !has_group) ctx->attach_event = ev_gemm[J & 3];
      st = slim_dgemm(ctx, "inv_panel_dgemm", 1, d);
      if (st != SLIM_OK) return st;
      if (has_window) {
        // the window of the first block of a group lies in the group to the left, which far() of the group
        // before this one also writes
        if (wstart < g0 && far_issued) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s1, ev_far[last_far_slot], 0));
        d.A = R + j0;                               // rows 0 .. jn of the panel
        d.lda = lda;
        d.B = R + (int64_t)wstart * lda + j0;       // rows of the panel that belong to the window
        d.ldb = lda;
        d.C = A + wstart;
        d.ldc = lda;
        d.M = jn;
        d.N = j0 - wstart;
        d.K = nbk;
        d.alpha = -1.0;
        d.beta = 1.0;
        if (!has_group) ctx->attach_event = ev_gemm[J & 3];
        st = slim_dgemm(ctx, "inv_window_dgemm", 1, d);
        if (st != SLIM_OK) return st;
      }
      if (has_group) {
        // every panel of the group except the first block's is complete: bring the group to the left up to date
        const int gp = g0 - GRP * NB;               // first column of the group to the left
        if (far_issued) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s1, ev_far[last_far_slot], 0));
        d.A = R + j0;                               // R[0:g0, j0:g1]
        d.lda = lda;
        d.B = R + (int64_t)gp * lda + j0;
        d.ldb = lda;
        d.C = A + gp;
        d.ldc = lda;
        d.M = g0;
        d.N = g0 - gp;
        d.K = g1 - j0;
        d.flags = 0;
        d.alpha = -1.0;
        d.beta = 1.0;
        ctx->attach_event = ev_gemm[J & 3];
        st = slim_dgemm(ctx, "inv_group_next_dgemm", 1, d);
        if (st != SLIM_OK) return st;
      }
      SLIM_HIP_TRY(ctx, slim_attach_flush(ctx));
    }
    // ---- s2: everything two or more groups to the left, once all panels of the group exist
    if (J == G * GRP && g0 - GRP * NB > 0) {
      StreamSwap swap(ctx, s2);
      const int gp = g0 - GRP * NB;
      SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s2, ev_gemm[J & 3], 0));
      slim_gemm_desc d;
      d.A = R + g0;                                 // R[0:gp, g0:g1]
      d.lda = lda;
      d.B = R + g0;
      d.ldb = lda;
      d.C = A;
      d.ldc = lda;
      d.C2 = nullptr;
      d.ldc2 = 0;
      d.M = gp;
      d.N = gp;
      d.K = g1 - g0;
      // While this update is short next to the four diagonal steps it runs beside, it runs as a persistent
      // kernel that leaves some CUs to their kernels; a large one is throughput-bound and takes the whole chip.
      d.flags = SLIM_GEMM_UPPER_ONLY | (gp <= 4096 ? SLIM_GEMM_ONE_PER_CU : 0);
      d.alpha = -1.0;
      d.beta = 1.0;
      last_far_slot ^= 1;
      ctx->attach_event = ev_far[last_far_slot];
      st = slim_dgemm(ctx, "inv_syrk_dgemm", 1, d);
      if (st != SLIM_OK) return st;
      SLIM_HIP_TRY(ctx, slim_attach_flush(ctx));
      far_issued = true;
    }
  }
  // The pivots are all known once the last diagonal block is done: the flag travels to the host from here, and the
  // call returns when it has arrived, with the triangular inverse still in flight on the stream.
  int* host = reinterpret_cast<int*>(ctx->hpin);
  hipEvent_t ev_info = ctx->ev[11];
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(host, flag, sizeof(int), hipMemcpyDeviceToHost, s0));
  SLIM_HIP_TRY(ctx, hipEventRecord(ev_info, s0));
  // the leftmost group's share of the triangular inverse: behind the last diagonal block and the last panels
  hipEvent_t ev_last = ctx->ev[15], ev_tri = ctx->ev[14];
  SLIM_HIP_TRY(ctx, hipEventRecord(ev_last, s0));
  SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s3, ev_last, 0));
  if (nblk > 1) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s3, ev_gemm[1 & 3], 0));
  st = group_inverse(0);
  if (st != SLIM_OK) return st;
  SLIM_HIP_TRY(ctx, hipEventRecord(ev_tri, s3));
  // every side stream has joined the caller's before the call's results are read (and before the workspace is reused)
  if (nblk > 1) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s0, ev_gemm[1 & 3], 0));
  if (far_issued) SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s0, ev_far[last_far_slot], 0));
  SLIM_HIP_TRY(ctx, hipStreamWaitEvent(s0, ev_tri, 0));

  SLIM_LAUNCH(ctx, "inv_diag_colsumsq", colsumsq_upper, dim3(slim_cdiv(m, 64), parts), dim3(256), 0, U, ldu, m, partial);
  SLIM_LAUNCH(ctx, "inv_diag_finalize", colsum_finalize, dim3(slim_cdiv(m, 256)), dim3(256), 0, partial, parts, m, hinv_diag);

  SLIM_HIP_TRY(ctx, hipEventSynchronize(ev_info));
  ctx->staging_copy_pending = false;               // the copy of the descriptors lies before the flag's on the stream
  *info = host[0];
  if (host[0] != 0)
    return slim_fail(ctx, SLIM_ERR_NOT_PD, "slim_hessian_inverse: H + lambda I is not positive definite (pivot at column %d)", host[0]);
  return SLIM_OK;
}
