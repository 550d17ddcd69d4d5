// a4  Salience-Determined Bit Allocation (Eq. 4; Alg. 2 SBA; App. C, App. D), all in fp64.
//
// The search evaluates floor(k/2)+1 allocations that differ from one another in two groups only, so the
// layer outputs are carried incrementally:
//   sba_rank        stable ascending rank of the k group saliences (one workgroup, counting sort by
//                   comparison; NaN ranks last) -> order[]
//   sba_fakequant   per (row, group), one wavefront: Eq. 1 / Eq. 2 round-to-nearest at width N and at the one
//                   other width the group can take; stores W_N and the difference, the latter in search order
//   dgemm           Y^T = W X_s and Y_0^T = W_N X_s     (n x t_s, fp64 matrix cores)
//   kl_ref_*        once: per token the maximum M_t and log-sum-exp of the reference outputs; Y is then overwritten
//                   by P = softmax(Y) and B_t = sum_i P_i log P_i is kept
//   for p = 0 .. floor(k/2):
//     kl_step / kl_finalize   obj[p] = sum_tokens KL(softmax(Y_t) || softmax(Y_p,t))
//                   = sum_t [ B_t - (sum_i P_i q_i - lse(q)) ]: ONE pass over P and Y_p per candidate, with the
//                   reference maximum M_t as the shift of the exponentials (Y_p differs from Y by quantisation
//                   noise, so M_t is as good a shift as the maximum of Y_p itself).  The softmax runs over the n
//                   outputs of a token, i.e. down a column of the transposed outputs, so consecutive lanes read
//                   consecutive tokens
//     dgemm         Y_{p+1}^T = Y_p^T + [D_lo(g_lo) | D_hi(g_hi)] [X_s(g_lo) ; X_s(g_hi)]  (rank 2 beta; the
//                   operands were laid out in search order on the device, no host round trip)
//   sba_finalize    first minimum of obj, bit vector of p*
#include <algorithm>

#include "dgemm_device.h"
#include "slim_device.h"
#include "slim_internal.h"

namespace {

using namespace slimdev;

constexpr int KL_TOK = 64;     // tokens per workgroup
constexpr int KL_PART = 5;     // doubles per (part, token): max y, sum exp y, sum P log P, sum exp q, sum P q (or squared error)

__global__ __launch_bounds__(256) void sba_rank(const double* __restrict__ sal, int k, int* __restrict__ order,
                                                int* __restrict__ rank_of) {
  for (int g = threadIdx.x; g < k; g += 256) {
    double v = sal[g];
    if (v != v) v = INFINITY;
    int rank = 0;
    for (int h = 0; h < k; ++h) {
      double u = sal[h];
      if (u != u) u = INFINITY;
      rank += (u < v || (u == v && h < g)) ? 1 : 0;
    }
    order[rank] = g;
    rank_of[g] = rank;
  }
}

// round-to-nearest fake quantisation of one value with the row-group's default parameters
struct RtnParams {
  double delta0, z, qmax, alpha;
  bool sign;
};

__device__ __forceinline__ RtnParams rtn_params(double mn, double mx, double mean_abs, int bits, int q1_mode) {
  RtnParams p;
  p.sign = (bits == 1 && q1_mode == SLIM_Q1_SIGN);
  p.alpha = mean_abs;
  p.qmax = (double)((1 << bits) - 1);
  p.delta0 = 1.0;
  p.z = 0.0;
  if (!p.sign) {
    if (mx == mn) {
      mn = fmin(mn, 0.0);
      mx = fmax(mx, 0.0);
    }
    if (mx != mn) {
      p.delta0 = (mx - mn) / p.qmax;
      p.z = -rint(mn / p.delta0);
    }
  }
  return p;
}

__device__ __forceinline__ double rtn_apply(const RtnParams& p, double w) {
  if (p.sign) return (w >= 0.0) ? p.alpha : -p.alpha;
  const double q = fmin(fmax(rint(w / p.delta0) + p.z, 0.0), p.qmax);
  return p.delta0 * (q - p.z);
}

// one wavefront per (row, group); grid = ceil(n * k / 4) workgroups of 4 wavefronts.
// W_N goes to WN in the natural layout.  The difference to the other width a group can take is stored in
// "search order": column block r (2 beta wide) of Dcat holds [W_{N-1} - W_N of the r-th least salient group |
// W_{N+1} - W_N of the r-th most salient group], so that step r of the search is ONE rank-2beta update.
// `parts` selects what is written: FQ_WN (needs no ranking), FQ_DCAT, or both.
enum { FQ_WN = 1, FQ_DCAT = 2 };
__global__ __launch_bounds__(256) void sba_fakequant(const double* __restrict__ W, int n, int m, int beta, int N,
                                                     int q1_mode, const int* __restrict__ rank_of, int pmax,
                                                     double* __restrict__ WN, double* __restrict__ Dcat, int parts) {
  const int lane = threadIdx.x & 63;
  const int k = m / beta;
  const int64_t unit = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= (int64_t)n * k) return;
  const int row = (int)(unit / k), g = (int)(unit % k);
  const int64_t base = (int64_t)row * m + (int64_t)g * beta;
  double mn = INFINITY, mx = -INFINITY, sabs = 0.0;
  for (int c = lane; c < beta; c += 64) {
    const double v = W[base + c];
    mn = fmin(mn, v);
    mx = fmax(mx, v);
    sabs += fabs(v);
  }
  mn = wave_min(mn);
  mx = wave_max(mx);
  sabs = wave_sum(sabs) / (double)beta;
  const RtnParams pn = rtn_params(mn, mx, sabs, N, q1_mode);
  if (!(parts & FQ_DCAT)) {
    for (int c = lane; c < beta; c += 64) WN[base + c] = rtn_apply(pn, W[base + c]);
    return;
  }
  const int pos = rank_of[g];
  const bool low = pos < pmax, high = pos >= k - pmax;
  const RtnParams po = rtn_params(mn, mx, sabs, low ? N - 1 : N + 1, q1_mode);
  const int64_t dbase = (int64_t)row * m + (low ? (int64_t)pos * 2 * beta : (int64_t)(k - 1 - pos) * 2 * beta + beta);
  for (int c = lane; c < beta; c += 64) {
    const double v = W[base + c];
    const double wn = rtn_apply(pn, v);
    if (parts & FQ_WN) WN[base + c] = wn;
    if (low || high) Dcat[dbase + c] = rtn_apply(po, v) - wn;
  }
}

// rows of X_s in search order: row block r (2 beta rows) = [rows of the r-th least salient group ; rows of the
// r-th most salient group]
__global__ __launch_bounds__(256) void sba_gather_x(const double* __restrict__ X64, int64_t ts, int beta, int k,
                                                    const int* __restrict__ order, double* __restrict__ Xcat) {
  const int r = blockIdx.y >> 1, h = blockIdx.y & 1;
  const int g = h ? order[k - 1 - r] : order[r];
  const int64_t total = (int64_t)beta * ts;
  const double* src = X64 + (int64_t)g * beta * ts;
  double* dst = Xcat + ((int64_t)r * 2 + h) * beta * ts;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 2; i < total; i += (int64_t)gridDim.x * 512)
    *reinterpret_cast<double2*>(dst + i) = *reinterpret_cast<const double2*>(src + i);
}

// ---- reference side, once per call ----------------------------------------------------------------
// grid (ceil(ts / 64), parts): 64 tokens x 4 row lanes per workgroup; part r owns rows [r*rpp, (r+1)*rpp).
// per (part, token): max y and sum exp(y - max)
__global__ __launch_bounds__(256) void kl_ref_partial(const double* __restrict__ Y, int n, int64_t ts, int rows_per_part,
                                                      double* __restrict__ partial) {
  __shared__ double red[2][4][KL_TOK];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * KL_TOK + tx;
  const int r0 = blockIdx.y * rows_per_part;
  const int r1 = min(n, r0 + rows_per_part);
  const bool live = t < ts;
  double my = -INFINITY;
  if (live)
    for (int r = r0 + ty; r < r1; r += 4) my = fmax(my, Y[(int64_t)r * ts + t]);
  red[0][ty][tx] = my;
  __syncthreads();
  my = fmax(fmax(red[0][0][tx], red[0][1][tx]), fmax(red[0][2][tx], red[0][3][tx]));
  double zy = 0.0;
  if (live && my > -INFINITY)
    for (int r = r0 + ty; r < r1; r += 4) zy += exp(Y[(int64_t)r * ts + t] - my);
  red[1][ty][tx] = zy;
  __syncthreads();
  if (ty == 0 && live) {
    double* o = partial + ((int64_t)blockIdx.y * ts + t) * KL_PART;
    o[0] = my;
    o[1] = ((red[1][0][tx] + red[1][1][tx]) + red[1][2][tx]) + red[1][3][tx];
  }
}

// one thread per token: merges the parts into tok[t] = {M_t, lse_t}
__global__ __launch_bounds__(256) void kl_ref_merge(const double* __restrict__ partial, int parts, int64_t ts,
                                                    double* __restrict__ tok) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= ts) return;
  double M = -INFINITY;
  for (int p = 0; p < parts; ++p) M = fmax(M, partial[((int64_t)p * ts + t) * KL_PART]);
  double Z = 0.0;
  for (int p = 0; p < parts; ++p) {
    const double* o = partial + ((int64_t)p * ts + t) * KL_PART;
    Z += o[1] * exp(o[0] - M);
  }
  tok[2 * t] = M;
  tok[2 * t + 1] = M + log(Z);
}

// Y <- P = exp(Y - lse); per (part, token) the partial sum of P log P goes to slot 2
__global__ __launch_bounds__(256) void kl_ref_softmax(double* __restrict__ Y, int n, int64_t ts, int rows_per_part,
                                                      const double* __restrict__ tok, double* __restrict__ partial) {
  __shared__ double red[4][KL_TOK];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * KL_TOK + tx;
  const int r0 = blockIdx.y * rows_per_part;
  const int r1 = min(n, r0 + rows_per_part);
  double b = 0.0;
  if (t < ts) {
    const double lse = tok[2 * t + 1];
    for (int r = r0 + ty; r < r1; r += 4) {
      const double lp = Y[(int64_t)r * ts + t] - lse;
      const double pr = exp(lp);
      Y[(int64_t)r * ts + t] = pr;
      b = fma(pr, lp, b);
    }
  }
  red[ty][tx] = b;
  __syncthreads();
  if (ty == 0 && t < ts)
    partial[((int64_t)blockIdx.y * ts + t) * KL_PART + 2] = ((red[0][tx] + red[1][tx]) + red[2][tx]) + red[3][tx];
}

// one thread per token: B_t = sum_i P_i log P_i (fixed order over the parts) into tok2[t]
__global__ __launch_bounds__(256) void kl_ref_entropy(const double* __restrict__ partial, int parts, int64_t ts,
                                                      double* __restrict__ tokB) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= ts) return;
  double b = 0.0;
  for (int p = 0; p < parts; ++p) b += partial[((int64_t)p * ts + t) * KL_PART + 2];
  tokB[t] = b;
}

// ---- per candidate -------------------------------------------------------------------------------------
// per (part, token): sum exp(q - M_t) and sum P q over the part's rows, one pass
__global__ __launch_bounds__(256) void kl_step(const double* __restrict__ P, const double* __restrict__ Q, int n,
                                               int64_t ts, int rows_per_part, const double* __restrict__ tok,
                                               double* __restrict__ partial) {
  __shared__ double red[2][4][KL_TOK];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * KL_TOK + tx;
  const int r0 = blockIdx.y * rows_per_part;
  const int r1 = min(n, r0 + rows_per_part);
  double z0 = 0.0, z1 = 0.0, a0 = 0.0, a1 = 0.0;
  if (t < ts) {
    const double M = tok[2 * t];
    int r = r0 + ty;
    for (; r + 4 < r1; r += 8) {
      const double q0 = Q[(int64_t)r * ts + t], q1 = Q[(int64_t)(r + 4) * ts + t];
      const double p0 = P[(int64_t)r * ts + t], p1 = P[(int64_t)(r + 4) * ts + t];
      z0 += exp(q0 - M);
      z1 += exp(q1 - M);
      a0 = fma(p0, q0, a0);
      a1 = fma(p1, q1, a1);
    }
    if (r < r1) {
      const double q0 = Q[(int64_t)r * ts + t];
      z0 += exp(q0 - M);
      a0 = fma(P[(int64_t)r * ts + t], q0, a0);
    }
  }
  red[0][ty][tx] = z0 + z1;
  red[1][ty][tx] = a0 + a1;
  __syncthreads();
  if (ty == 0 && t < ts) {
    double* o = partial + ((int64_t)blockIdx.y * ts + t) * KL_PART;
    o[3] = ((red[0][0][tx] + red[0][1][tx]) + red[0][2][tx]) + red[0][3][tx];
    o[4] = ((red[1][0][tx] + red[1][1][tx]) + red[1][2][tx]) + red[1][3][tx];
  }
}

// one thread per token: KL_t = B_t - (sum P q - (M_t + log sum exp(q - M_t))); every workgroup of 256 tokens
// writes its sum
__global__ __launch_bounds__(256) void kl_finalize(const double* __restrict__ partial_all, int64_t pstride, int parts,
                                                   int64_t ts, const double* __restrict__ tok,
                                                   const double* __restrict__ tokB, double* __restrict__ block_sums_all,
                                                   int nblocks) {
  __shared__ double red[256];
  const double* partial = partial_all + (int64_t)blockIdx.y * pstride;       // blockIdx.y = candidate
  double* block_sums = block_sums_all + (int64_t)blockIdx.y * nblocks;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  double acc = 0.0;
  if (t < ts) {
    double Z = 0.0, A = 0.0;
    for (int p = 0; p < parts; ++p) {
      const double* o = partial + ((int64_t)p * ts + t) * KL_PART;
      Z += o[3];
      A += o[4];
    }
    acc = tokB[t] - (A - (tok[2 * t] + log(Z)));
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int st = 128; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) block_sums[blockIdx.x] = red[0];
}

// squared-error objective: per (part, token) the sum over the part's rows of (y - q)^2, stored in slot 4 of the
// same partial layout so that the fixed-order reductions are shared
__global__ __launch_bounds__(256) void mse_partial(const double* __restrict__ Y, const double* __restrict__ Q, int n,
                                                   int64_t ts, int rows_per_part, double* __restrict__ partial) {
  __shared__ double red[4][KL_TOK];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * KL_TOK + tx;
  const int r0 = blockIdx.y * rows_per_part;
  const int r1 = min(n, r0 + rows_per_part);
  double a = 0.0;
  if (t < ts) {
    for (int r = r0 + ty; r < r1; r += 4) {
      const double dlt = Y[(int64_t)r * ts + t] - Q[(int64_t)r * ts + t];
      a = fma(dlt, dlt, a);
    }
  }
  red[ty][tx] = a;
  __syncthreads();
  if (ty == 0 && t < ts) partial[((int64_t)blockIdx.y * ts + t) * KL_PART + 4] = ((red[0][tx] + red[1][tx]) + red[2][tx]) + red[3][tx];
}

// one thread per token: sums the row parts of its token; every workgroup of 256 tokens writes its sum
__global__ __launch_bounds__(256) void mse_finalize(const double* __restrict__ partial_all, int64_t pstride, int parts,
                                                    int64_t ts, double* __restrict__ block_sums_all, int nblocks) {
  __shared__ double red[256];
  const double* partial = partial_all + (int64_t)blockIdx.y * pstride;       // blockIdx.y = candidate
  double* block_sums = block_sums_all + (int64_t)blockIdx.y * nblocks;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  double acc = 0.0;
  if (t < ts)
    for (int p = 0; p < parts; ++p) acc += partial[((int64_t)p * ts + t) * KL_PART + 4];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int st = 128; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) block_sums[blockIdx.x] = red[0];
}

// obj[p] = sum of the token-block sums of step p (fixed order); then the first minimum and its bit vector
__global__ __launch_bounds__(256) void sba_finalize(const double* __restrict__ block_sums, int nblocks,
                                                    double* __restrict__ obj, int pmax, const int* __restrict__ order,
                                                    int k, int N, uint8_t* __restrict__ bits, int* __restrict__ p_star) {
  __shared__ int best_p;
  for (int p = threadIdx.x; p <= pmax; p += 256) {
    double s = 0.0;
    for (int w = 0; w < nblocks; ++w) s += block_sums[(int64_t)p * nblocks + w];
    obj[p] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int bp = 0;
    double bv = obj[0];
    for (int p = 1; p <= pmax; ++p) {
      if (obj[p] < bv) {
        bv = obj[p];
        bp = p;
      }
    }
    best_p = bp;
    *p_star = bp;
  }
  __syncthreads();
  const int ps = best_p;
  for (int r = threadIdx.x; r < k; r += 256) {
    int b = N;
    if (r < ps) b = N - 1;
    if (r >= k - ps) b = N + 1;
    bits[order[r]] = (uint8_t)b;
  }
}

}  // namespace

namespace {

// ---- the whole search in one kernel -----------------------------------------------------------------
// One workgroup per 128 x 128 tile of the outputs (rows x tokens) keeps the tile of the current candidate's
// outputs in its accumulator registers from the first candidate to the last: per candidate it adds the tile's
// terms of the objective (per token: sum exp(q - M) and sum P q over the tile's rows, or the squared error)
// to the candidate's partials and then applies the rank-2beta update of the next candidate on the matrix cores
// (the K loop of the fp64 GEMM).  The candidates' outputs never go back to memory: per candidate the kernel reads
// the reference tile once and two thin operand slabs, where a GEMM launch per candidate reads and writes all
// outputs and a second kernel reads them again.
struct SearchArgs {
  const double* Yc;        // n x ts outputs of the all-N-bit weights
  const double* R;         // n x ts reference: P = softmax(Y) (KL) or Y (squared error)
  const double* tok;       // per token {max, log-sum-exp} of the reference (KL)
  const double* Dcat;      // n x m, column block p: the change of W from candidate p to p + 1
  const double* Xcat;      // m x ts, row block p: the rows of X_s that change meets
  double* partial;         // per candidate (stride pstride) [row block][token][KL_PART]
  int64_t pstride, ts;
  int n, m, beta, pmax;
};

constexpr int SEARCH_TILE = 128;
constexpr size_t SEARCH_LDS = sizeof(double) * (2 * (slimgemm::BK * SEARCH_TILE * 2) + 4 * SEARCH_TILE);

template <int OBJ>
__global__ __launch_bounds__(256, 2) void sba_search_tile(SearchArgs a) {   // two wavefronts per SIMD
  using namespace slimgemm;
  constexpr int BM = SEARCH_TILE, BN = SEARCH_TILE, MI = 4, NJ = 4;
  extern __shared__ __align__(16) double smem[];
  double* red = smem + 2 * (BK * BM + BK * BN);        // [sum exp | sum P q][upper | lower 64 rows][128 tokens]
  const int tiles_n = (int)(a.ts / BN);
  const int bi = blockIdx.x / tiles_n, bj = blockIdx.x % tiles_n;
  const int row0 = bi * BM, col0 = bj * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, l16 = lane & 15, lk = lane >> 4;
  // accumulator register v of tile (i, j) of this lane is row 16 i + 4 v + lk, column 16 j + l16 of the wavefront's
  // 64 x 64 quarter
  const int64_t ts = a.ts;
  const int rbase = row0 + wm * 64 + lk, cbase = col0 + wn * 64 + l16;
  double4v acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j][v] = a.Yc[(int64_t)(rbase + 16 * i + 4 * v) * ts + cbase + 16 * j];
  double Mt[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) Mt[j] = (OBJ == SLIM_OBJ_KL) ? a.tok[2 * (int64_t)(cbase + 16 * j)] : 0.0;

  for (int p = 0; p <= a.pmax; ++p) {
    double z[NJ], s[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) z[j] = s[j] = 0.0;
    // The addresses of the reference tile are formed again for every candidate from this pointer (opaque to the
    // compiler): kept across the K loop below they would cost 32 registers and spill.
    const double* rtile = a.R + (int64_t)rbase * ts + cbase;
    asm volatile("" : "+v"(rtile));
    // (the condition always holds; as a block of its own this part is register-allocated apart from the K loop,
    // and the kernel no longer spills)
    if (a.n > 0)
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      // 16 reference values in flight at a time: all 64 would not leave room for two workgroups per CU
      double ref[4][NJ];
#pragma unroll
      for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int j = 0; j < NJ; ++j) ref[v][j] = rtile[(int64_t)(16 * i + 4 * v) * ts + 16 * j];
#pragma unroll
      for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const double q = acc[i][j][v];
          if (OBJ == SLIM_OBJ_KL) {
            z[j] += exp(q - Mt[j]);
            s[j] = fma(ref[v][j], q, s[j]);
          } else {
            const double dlt = ref[v][j] - q;
            s[j] = fma(dlt, dlt, s[j]);
          }
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the four lanes that share a token column, then the two wavefronts that do
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      z[j] += shfl_xor_f64(z[j], 16);
      z[j] += shfl_xor_f64(z[j], 32);
      s[j] += shfl_xor_f64(s[j], 16);
      s[j] += shfl_xor_f64(s[j], 32);
      if (lk == 0) {
        red[(0 * 2 + wm) * BN + wn * 64 + 16 * j + l16] = z[j];
        red[(1 * 2 + wm) * BN + wn * 64 + 16 * j + l16] = s[j];
      }
    }
    __syncthreads();
    if (tid < BN) {
      double* o = a.partial + (int64_t)p * a.pstride + ((int64_t)bi * ts + col0 + tid) * KL_PART;
      o[3] = red[0 * BN + tid] + red[1 * BN + tid];
      o[4] = red[2 * BN + tid] + red[3 * BN + tid];
    }
    if (p == a.pmax) break;
    // candidate p + 1: Y^T += [D_lo | D_hi]_p [X_lo ; X_hi]_p, a rank-2beta update of the tile
    slim_gemm_desc d;
    d.A = a.Dcat + (int64_t)p * 2 * a.beta;
    d.lda = a.m;
    d.B = a.Xcat + (int64_t)p * 2 * a.beta * ts;
    d.ldb = ts;
    k_loop_fast<0, BM, BN>(d, row0, col0, 0, 2 * a.beta, smem, acc);
  }
}

}  // namespace

namespace {

// The workspace of slim_sba_allocate; slim_sba_prepare fills the part of it that does not depend on the ranking.
struct SbaWorkspace {
  bool fused;            // the search runs as one kernel over 128 x 128 output tiles
  int k, pmax, rpp, parts, kl_blocks;
  int64_t pstride;
  double *W64, *WN, *Dcat, *X64, *Xcat, *Yt, *Yc, *partial, *obj, *block_sums, *tok, *tokB;
  int *order, *rank_of, *pstar_dev;
};

}  // namespace

size_t slim_ws_need_sba(int n, int m, int beta, int64_t t_s) {
  const int k = m / beta, pmax = k / 2;
  const bool fused = n % SEARCH_TILE == 0 && t_s % SEARCH_TILE == 0 && (2 * beta) % 16 == 0;
  const int parts = slim_cdiv(n, fused ? SEARCH_TILE : 256), kl_blocks = slim_cdiv(t_s, 256);
  const size_t bW = slim_ws_round(sizeof(double) * (size_t)n * m);
  const size_t bX = slim_ws_round(sizeof(double) * (size_t)m * t_s);
  const size_t bY = slim_ws_round(sizeof(double) * (size_t)n * t_s);
  const size_t bPart = slim_ws_round(sizeof(double) * (size_t)parts * t_s * KL_PART);
  const size_t bObj = slim_ws_round(sizeof(double) * (size_t)(pmax + 2) * (size_t)(kl_blocks + 1));
  const size_t bOrd = slim_ws_round(sizeof(int) * (size_t)(2 * k + 2));
  const size_t bTok = slim_ws_round(sizeof(double) * 3 * (size_t)t_s);
  return 3 * bW + 2 * bX + 2 * bY + (size_t)(pmax + 1) * bPart + bObj + bOrd + bTok + 256;
}

namespace {

slim_status sba_workspace(slim_ctx* ctx, int n, int m, int beta, int64_t t_s, SbaWorkspace& w) {
  w.k = m / beta;
  w.pmax = w.k / 2;
  // The one-kernel search needs whole tiles and whole K slabs; its partials are per 128 rows.
  w.fused = n % SEARCH_TILE == 0 && t_s % SEARCH_TILE == 0 && (2 * beta) % 16 == 0;
  w.rpp = w.fused ? SEARCH_TILE : 256;                  // rows per part of the reduction over the outputs
  w.parts = slim_cdiv(n, w.rpp);
  w.kl_blocks = slim_cdiv(t_s, 256);
  const size_t bW = slim_ws_round(sizeof(double) * (size_t)n * m);
  const size_t bX = slim_ws_round(sizeof(double) * (size_t)m * t_s);
  const size_t bY = slim_ws_round(sizeof(double) * (size_t)n * t_s);
  const size_t bPart = slim_ws_round(sizeof(double) * (size_t)w.parts * t_s * KL_PART);   // per candidate
  const size_t bObj = slim_ws_round(sizeof(double) * (size_t)(w.pmax + 2) * (size_t)(w.kl_blocks + 1));
  const size_t bOrd = slim_ws_round(sizeof(int) * (size_t)(2 * w.k + 2));
  const size_t bTok = slim_ws_round(sizeof(double) * 3 * (size_t)t_s);
  slim_status st = slim_ws_reserve(ctx, slim_ws_need_sba(n, m, beta, t_s));
  if (st != SLIM_OK) return st;
  w.W64 = static_cast<double*>(slim_ws_alloc(ctx, bW));
  w.WN = static_cast<double*>(slim_ws_alloc(ctx, bW));
  w.Dcat = static_cast<double*>(slim_ws_alloc(ctx, bW));
  w.X64 = static_cast<double*>(slim_ws_alloc(ctx, bX));
  w.Xcat = static_cast<double*>(slim_ws_alloc(ctx, bX));
  w.Yt = static_cast<double*>(slim_ws_alloc(ctx, bY));
  w.Yc = static_cast<double*>(slim_ws_alloc(ctx, bY));
  w.partial = static_cast<double*>(slim_ws_alloc(ctx, (size_t)(w.pmax + 1) * bPart));
  w.pstride = (int64_t)(bPart / sizeof(double));        // every candidate keeps its partials until the end
  w.obj = static_cast<double*>(slim_ws_alloc(ctx, bObj));
  w.block_sums = w.obj + (w.pmax + 2);
  w.order = static_cast<int*>(slim_ws_alloc(ctx, bOrd));
  w.rank_of = w.order + (w.k + 1);
  w.pstar_dev = static_cast<int*>(slim_ws_alloc(ctx, 256));
  w.tok = static_cast<double*>(slim_ws_alloc(ctx, bTok));   // per token {max, log-sum-exp} of the reference
  w.tokB = w.tok + 2 * t_s;                                 // per token sum P log P
  return SLIM_OK;
}

slim_status sba_check(slim_ctx* ctx, const char* fn, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                      int beta, int N, int objective, const void* X_s, slim_dtype x_dtype, int64_t t_s, int64_t ldxs,
                      const slim_params& prm) {
  SLIM_REQUIRE(ctx, W && X_s, "%s: null pointer", fn);
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "%s: need n, m > 0 and beta | m", fn);
  SLIM_REQUIRE(ctx, N >= 2 && N <= 7, "%s: N must be in 2..7 (got %d)", fn, N);
  SLIM_REQUIRE(ctx, beta % 4 == 0 && ldw >= m && ldw % 4 == 0, "%s: beta and ldw must be multiples of 4", fn);
  SLIM_REQUIRE(ctx, t_s > 0 && t_s % 4 == 0 && ldxs >= t_s && ldxs % 4 == 0,
               "%s: t_s and ldxs must be positive multiples of 4", fn);
  SLIM_REQUIRE(ctx, slim_aligned16(W) && slim_aligned16(X_s), "%s: misaligned pointer", fn);
  SLIM_REQUIRE(ctx, prm.q1_mode == 0 || prm.q1_mode == 1, "%s: unknown q1_mode", fn);
  SLIM_REQUIRE(ctx, objective == SLIM_OBJ_KL || objective == SLIM_OBJ_MSE, "%s: unknown objective %d", fn, objective);
  if (w_dtype == SLIM_F64 || x_dtype == SLIM_F64 || x_dtype == SLIM_F32)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "%s: W must be F16/BF16/F32 and X_s F16/BF16", fn);
  SLIM_REQUIRE(ctx, (size_t)(m / beta / 2 + 2) * sizeof(double) <= (size_t)SLIM_HPIN_BYTES, "%s: too many groups", fn);
  return SLIM_OK;
}

// The part of the objective that does not depend on the ranking (Eq. 4): W and X_s in fp64, the all-N-bit weights,
// the reference outputs Y^T = W X_s and the outputs of the all-N-bit weights, and for the KL objective the reference
// softmax with its per-token statistics.  `beside_chain` runs the two products in the form that leaves CUs free.
slim_status sba_rank_independent(slim_ctx* ctx, const SbaWorkspace& w, const void* W, slim_dtype w_dtype, int n, int m,
                                 int64_t ldw, int beta, int N, int objective, const void* X_s, slim_dtype x_dtype,
                                 int64_t t_s, int64_t ldxs, int q1_mode, bool beside_chain) {
  slim_status st = slim_widen_f64(ctx, "sba_widen_w", W, w_dtype, n, m, ldw, w.W64, (int64_t)m);
  if (st != SLIM_OK) return st;
  st = slim_widen_f64(ctx, "sba_widen_x", X_s, x_dtype, m, (int)t_s, ldxs, w.X64, t_s);
  if (st != SLIM_OK) return st;
  SLIM_LAUNCH(ctx, "sba_fakequant", sba_fakequant, dim3(slim_cdiv((int64_t)n * w.k, 4)), dim3(256), 0, w.W64, n, m, beta,
              N, q1_mode, nullptr, w.pmax, w.WN, nullptr, FQ_WN);
  slim_gemm_desc d;
  d.A = w.W64;
  d.lda = m;
  d.B = w.X64;
  d.ldb = t_s;
  d.C = w.Yt;
  d.ldc = t_s;
  d.C2 = nullptr;
  d.ldc2 = 0;
  d.M = n;
  d.N = (int)t_s;
  d.K = m;
  d.flags = 0;
  d.alpha = 1.0;
  d.beta = 0.0;
  slim_gemm_desc pair[2] = {d, d};
  pair[1].A = w.WN;
  pair[1].C = w.Yc;
  // Beside the inverse only as many rows of the two products run (persistent, on part of the chip) as take about
  // as long as the inverse does; the rest follows in the ordinary form, which wants the whole chip.  The inverse
  // is modelled as its chain of m / 64 diagonal steps of 45 us plus m^3 / 3 flops of triangular inversion at
  // 50 TFLOP/s, the persistent form at 85 % of the matrix cores of its CUs.
  // Their share of the chip, next to a factorisation whose own bulk updates want whole CUs too: 5/8 when the layer
  // has no more outputs than inputs (the products are then about as long as the inverse, and a larger share ends
  // them with it), half of it otherwise (most of the products follows after the inverse anyway, and the inverse
  // gains more from the CUs); both measured, on 4096 x 4096 .. 28672 x 8192 layers.
  int rows_beside = 0;
  const int cus = std::max(1, n <= m ? ctx->num_cus * 5 / 8 : ctx->num_cus / 2);
  if (beside_chain && n % 256 == 0 && t_s % 128 == 0 && m % 16 == 0) {
    const double t_inv = (m / 64) * 45e-6 + (double)m * m * m / 3.0 / 50e12;
    const double rate = 0.85 * 78.6e12 * cus / std::max(1, ctx->num_cus);
    const int64_t tiles_per_block = 2 * (t_s / 128);            // of 256 rows, both products
    int64_t tiles_fit = (int64_t)(rate * t_inv / (2.0 * 256 * 128 * m));
    tiles_fit = (tiles_fit / cus) * cus;                          // whole rounds
    rows_beside = (int)std::min<int64_t>(n, std::max<int64_t>(tiles_fit / tiles_per_block, 0) * 256);
  }
  if (rows_beside > 0) {
    slim_gemm_desc part[2] = {pair[0], pair[1]};
    part[0].M = part[1].M = rows_beside;
    st = slim_dgemm_reserved(ctx, "sba_output_dgemm", 0, part, 2, cus);
    if (st != SLIM_OK) return st;
  }
  if (rows_beside < n) {
    for (slim_gemm_desc g : pair) {
      g.A += (int64_t)rows_beside * g.lda;
      g.C += (int64_t)rows_beside * g.ldc;
      g.M = n - rows_beside;
      st = slim_dgemm(ctx, "sba_output_dgemm", 0, g);
      if (st != SLIM_OK) return st;
    }
  }
  if (objective == SLIM_OBJ_KL) {
    // reference side once: per-token maximum and log-sum-exp, then Y^T becomes P = softmax over the outputs
    const dim3 kgrid(slim_cdiv(t_s, KL_TOK), w.parts);
    SLIM_LAUNCH(ctx, "sba_kl_ref", kl_ref_partial, kgrid, dim3(256), 0, w.Yt, n, t_s, w.rpp, w.partial);
    SLIM_LAUNCH(ctx, "sba_kl_ref", kl_ref_merge, dim3(w.kl_blocks), dim3(256), 0, w.partial, w.parts, t_s, w.tok);
    SLIM_LAUNCH(ctx, "sba_kl_ref", kl_ref_softmax, kgrid, dim3(256), 0, w.Yt, n, t_s, w.rpp, w.tok, w.partial);
    SLIM_LAUNCH(ctx, "sba_kl_ref", kl_ref_entropy, dim3(w.kl_blocks), dim3(256), 0, w.partial, w.parts, t_s, w.tokB);
  }
  return SLIM_OK;
}

}  // namespace

extern "C" slim_status slim_sba_prepare(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                                        int beta, int N, int objective, const void* X_s, slim_dtype x_dtype,
                                        int64_t t_s, int64_t ldxs, const slim_params* params) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  slim_params prm;
  slim_default_params(&prm);
  if (params) prm = *params;
  slim_status st = sba_check(ctx, "slim_sba_prepare", W, w_dtype, n, m, ldw, beta, N, objective, X_s, x_dtype, t_s, ldxs, prm);
  if (st != SLIM_OK) return st;
  SbaWorkspace w;
  st = sba_workspace(ctx, n, m, beta, t_s, w);
  if (st != SLIM_OK) return st;
  st = sba_rank_independent(ctx, w, W, w_dtype, n, m, ldw, beta, N, objective, X_s, x_dtype, t_s, ldxs, prm.q1_mode, true);
  if (st != SLIM_OK) return st;
  slim_sba_prepared& r = ctx->sba_prep;
  r.W = W;
  r.X_s = X_s;
  r.ws = ctx->ws;
  r.w_dtype = w_dtype;
  r.x_dtype = x_dtype;
  r.n = n;
  r.m = m;
  r.beta = beta;
  r.N = N;
  r.objective = objective;
  r.q1_mode = prm.q1_mode;
  r.ldw = ldw;
  r.t_s = t_s;
  r.ldxs = ldxs;
  r.valid = true;
  return SLIM_OK;
}

extern "C" slim_status slim_sba_allocate(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                                         const double* group_sal, int beta, int N, int objective, const void* X_s,
                                         slim_dtype x_dtype, int64_t t_s, int64_t ldxs, const slim_params* params,
                                         uint8_t* bits, int* p_star, double* obj_curve) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  slim_params prm;
  slim_default_params(&prm);
  if (params) prm = *params;
  SLIM_REQUIRE(ctx, group_sal && bits, "slim_sba_allocate: null pointer");
  slim_status st = sba_check(ctx, "slim_sba_allocate", W, w_dtype, n, m, ldw, beta, N, objective, X_s, x_dtype, t_s, ldxs, prm);
  if (st != SLIM_OK) return st;
  // a preceding slim_sba_prepare with the same arguments has left the rank-independent part in the workspace
  const slim_sba_prepared r = ctx->sba_prep;
  const bool prepared = r.valid && r.W == W && r.X_s == X_s && r.w_dtype == (int)w_dtype && r.x_dtype == (int)x_dtype &&
                        r.n == n && r.m == m && r.beta == beta && r.N == N && r.objective == objective &&
                        r.q1_mode == prm.q1_mode && r.ldw == ldw && r.t_s == t_s && r.ldxs == ldxs;
  SbaWorkspace w;
  st = sba_workspace(ctx, n, m, beta, t_s, w);
  if (st != SLIM_OK) return st;
  const int k = w.k, pmax = w.pmax, rpp = w.rpp, parts = w.parts, kl_blocks = w.kl_blocks;
  const int64_t pstride = w.pstride;
  double *W64 = w.W64, *WN = w.WN, *Dcat = w.Dcat, *X64 = w.X64, *Xcat = w.Xcat, *Yt = w.Yt, *Yc = w.Yc;
  double *partial = w.partial, *obj = w.obj, *block_sums = w.block_sums, *tok = w.tok, *tokB = w.tokB;
  int *order = w.order, *rank_of = w.rank_of, *pstar_dev = w.pstar_dev;

  const bool reuse = prepared && r.ws == ctx->ws;       // (the workspace was not reallocated in between)
  if (!reuse) {
    st = sba_rank_independent(ctx, w, W, w_dtype, n, m, ldw, beta, N, objective, X_s, x_dtype, t_s, ldxs, prm.q1_mode, false);
    if (st != SLIM_OK) return st;
  }
  SLIM_LAUNCH(ctx, "sba_rank", sba_rank, dim3(1), dim3(256), 0, group_sal, k, order, rank_of);
  SLIM_LAUNCH(ctx, "sba_fakequant", sba_fakequant, dim3(slim_cdiv((int64_t)n * k, 4)), dim3(256), 0, W64, n, m, beta, N,
              prm.q1_mode, rank_of, pmax, WN, Dcat, FQ_DCAT);
  if (pmax > 0)
    SLIM_LAUNCH(ctx, "sba_gather_x", sba_gather_x, dim3(64, 2 * pmax), dim3(256), 0, X64, t_s, beta, k, order, Xcat);

  const dim3 kgrid(slim_cdiv(t_s, KL_TOK), parts);
  if (w.fused) {
    SearchArgs sa;
    sa.Yc = Yc;
    sa.R = Yt;
    sa.tok = tok;
    sa.Dcat = Dcat;
    sa.Xcat = Xcat;
    sa.partial = partial;
    sa.pstride = pstride;
    sa.ts = t_s;
    sa.n = n;
    sa.m = m;
    sa.beta = beta;
    sa.pmax = pmax;
    static bool lds_kl = false, lds_mse = false;
    const dim3 sgrid((n / SEARCH_TILE) * (int)(t_s / SEARCH_TILE));
    if (objective == SLIM_OBJ_KL) {
      if (!lds_kl) {
        SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(sba_search_tile<SLIM_OBJ_KL>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)SEARCH_LDS));
        lds_kl = true;
      }
      SLIM_LAUNCH(ctx, "sba_search", sba_search_tile<SLIM_OBJ_KL>, sgrid, dim3(256), SEARCH_LDS, sa);
    } else {
      if (!lds_mse) {
        SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(sba_search_tile<SLIM_OBJ_MSE>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)SEARCH_LDS));
        lds_mse = true;
      }
      SLIM_LAUNCH(ctx, "sba_search", sba_search_tile<SLIM_OBJ_MSE>, sgrid, dim3(256), SEARCH_LDS, sa);
    }
  } else {
    for (int p = 0; p <= pmax; ++p) {
      if (objective == SLIM_OBJ_KL)
        SLIM_LAUNCH(ctx, "sba_kl_step", kl_step, kgrid, dim3(256), 0, Yt, Yc, n, t_s, rpp, tok, partial + p * pstride);
      else
        SLIM_LAUNCH(ctx, "sba_mse_partial", mse_partial, kgrid, dim3(256), 0, Yt, Yc, n, t_s, rpp, partial + p * pstride);
      if (p < pmax) {
        // Y_{p+1}^T = Y_p^T + [D_lo | D_hi]_p [X_lo ; X_hi]_p : one rank-2beta update
        slim_gemm_desc u;
        u.A = Dcat + (int64_t)p * 2 * beta;
        u.lda = m;
        u.B = Xcat + (int64_t)p * 2 * beta * t_s;
        u.ldb = t_s;
        u.C = Yc;
        u.ldc = t_s;
        u.C2 = nullptr;
        u.ldc2 = 0;
        u.M = n;
        u.N = (int)t_s;
        u.K = 2 * beta;
        u.flags = 0;
        u.alpha = 1.0;
        u.beta = 1.0;
        st = slim_dgemm(ctx, "sba_update_dgemm", 0, u);
        if (st != SLIM_OK) return st;
      }
    }
  }
  // the per-token merges of all candidates in one launch (grid.y = candidate)
  if (objective == SLIM_OBJ_KL)
    SLIM_LAUNCH(ctx, "sba_kl_finalize", kl_finalize, dim3(kl_blocks, pmax + 1), dim3(256), 0, partial, pstride, parts, t_s,
                tok, tokB, block_sums, kl_blocks);
  else
    SLIM_LAUNCH(ctx, "sba_mse_finalize", mse_finalize, dim3(kl_blocks, pmax + 1), dim3(256), 0, partial, pstride, parts,
                t_s, block_sums, kl_blocks);
  SLIM_LAUNCH(ctx, "sba_finalize", sba_finalize, dim3(1), dim3(256), 0, block_sums, kl_blocks, obj, pmax, order, k, N,
              bits, pstar_dev);

  if (!p_star && !obj_curve) return SLIM_OK;       // nothing for the host: the call does not wait
  double* host_obj = reinterpret_cast<double*>(ctx->hpin);
  int* host_p = reinterpret_cast<int*>(ctx->hpin + sizeof(double) * (size_t)(pmax + 1));
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(host_obj, obj, sizeof(double) * (pmax + 1), hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(host_p, pstar_dev, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  if (p_star) *p_star = *host_p;
  if (obj_curve) memcpy(obj_curve, host_obj, sizeof(double) * (pmax + 1));
  return SLIM_OK;
}
