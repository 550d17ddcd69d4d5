// a5 - a8  3-sigma mask, Salience-Weighted Quantizer Calibration and the GPTQ-style column sweep
// (Sec. 3.3.2; Eq. 1, 2, 5; Alg. 1 lines 5-13; Alg. 2 SQC).
//
// Everything here is fp64: the rounding decisions of a sequential, error-feeding sweep only agree
// with a float64 reference if the working copy of W, the quantiser parameters and the compensation
// are carried at that precision.  CDNA4 runs fp64 vector and matrix work at full rate, so this
// costs little next to the Hessian.
//
// Per group of beta columns four kernels run back to back on the stream:
//   block_stats   shifted sums of the current block (for the block-wide 3-sigma rule), per row slab
//   sqc_search_fast / sqc_search_weighted   a few rows per workgroup: row min/max/mean|w|, the mask or the loss
//                 weights, then a few lanes per (row, 4 or 5 candidates) walk the row's weights in LDS;
//                 wavefront argmin with ties to the lower candidate index
//   gptq_sweep4   four rows per wavefront (16 lanes each), the row's beta weights in registers, the
//                 beta x beta block of U in LDS; beta serial steps of quantise -> error -> rank-1 update
//   dgemm         W[:, later] -= E_b U[b, later] on the fp64 matrix cores
#include <algorithm>
#include <utility>

#include "slim_device.h"
#include "slim_internal.h"

namespace {

using namespace slimdev;

constexpr int SQC_CPT = 4;        // candidates per thread in sqc_search_weighted
constexpr int SQC_THREADS = 256;
constexpr int STAT_ROWS = 8;      // rows per workgroup in block_stats
constexpr int GPTQ_WINC = 512;    // columns per window of the sweep's two-level trailing updates

// ------------------------------------------------------------------------------------------
// Shifted first and second moments of an n x beta block, one partial pair per slab of STAT_ROWS rows.
// The shift (the block's first element) keeps sigma^2 = E[(w-s)^2] - E[w-s]^2 well conditioned.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void block_stats(const double* __restrict__ W, int64_t ldw, int n, int beta,
                                                   double* __restrict__ partial) {
  __shared__ double red[2][4];
  const double shift = W[0];
  const int r0 = blockIdx.x * STAT_ROWS;
  const int rows = min(STAT_ROWS, n - r0);
  double s1 = 0.0, s2 = 0.0;
  for (int idx = threadIdx.x; idx < rows * beta; idx += 256) {
    const int r = idx / beta, c = idx - r * beta;
    const double d = W[(int64_t)(r0 + r) * ldw + c] - shift;
    s1 += d;
    s2 += d * d;
  }
  s1 = wave_sum(s1);
  s2 = wave_sum(s2);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    red[0][wave] = s1;
    red[1][wave] = s2;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    partial[2 * blockIdx.x] = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
    partial[2 * blockIdx.x + 1] = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];
  }
}

struct SqcArgs {
  const double* W;       // n x beta block of current weights
  int64_t ldw;
  int n, beta, bits;
  const double* omega;   // explicit weights (n x beta, ld = beta) or null
  const double* dblk;    // [H^-1]_jj of the block's columns (ELEMENT weights) or null
  const double* stat_partial;  // block_stats output or null (ROW scope / no mask needed)
  int nstat;
  int weight_mode, scope, q1_mode;
  const double* tau;
  int ncand;
  int rows_per_wg;       // rows of the block one workgroup calibrates
  double* scale;         // element i at scale[i * out_stride]
  double* zero;
  int64_t out_stride;
  int* cand_idx;         // optional, same stride
};

// Eq. 1 parameters of one row; identical operation order to the reference definition.
__device__ __forceinline__ void minmax_params(double wmin, double wmax, int bits, double& delta0, double& z) {
  const double qmax = (double)((1 << bits) - 1);
  if (wmax == wmin) {
    wmin = fmin(wmin, 0.0);
    wmax = fmax(wmax, 0.0);
  }
  if (wmax == wmin) {
    delta0 = 1.0;
    z = 0.0;
    return;
  }
  delta0 = (wmax - wmin) / qmax;
  z = -rint(wmin / delta0);
}

// sqc_search_weighted: the candidate search with a loss weight per element (explicit weights, or
// omega = w^2 / [H^-1]_jj^2), which the weights and the losses of a row pass through LDS for.
__global__ __launch_bounds__(SQC_THREADS) void sqc_search_weighted(SqcArgs a) {
  extern __shared__ __align__(16) double smem[];
  const int beta = a.beta, ncand = a.ncand;
  const int RW = a.rows_per_wg;
  double* wrow = smem;                            // [RW][beta]
  double* om = wrow + RW * beta;                  // [RW][beta]
  double* loss = om + RW * beta;                  // [RW][ncand]
  double* rp = loss + RW * ncand;                 // [RW][4]: delta0, z, alpha, unused
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r0 = blockIdx.x * RW;
  const int rows = min(RW, a.n - r0);
  const bool sign_mode = (a.bits == 1 && a.q1_mode == SLIM_Q1_SIGN);

  for (int idx = tid; idx < rows * beta; idx += SQC_THREADS) {
    const int r = idx / beta, c = idx - r * beta;
    wrow[r * beta + c] = a.W[(int64_t)(r0 + r) * a.ldw + c];
  }
  __syncthreads();

  // per-row statistics and loss weights: wavefront w takes rows w, w + 4
  for (int r = wave; r < rows; r += SQC_THREADS / 64) {
    const double* w = wrow + r * beta;
    double mn = INFINITY, mx = -INFINITY, sabs = 0.0;
    for (int c = lane; c < beta; c += 64) {
      const double v = w[c];
      mn = fmin(mn, v);
      mx = fmax(mx, v);
      sabs += fabs(v);
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    sabs = wave_sum(sabs);
    if (lane == 0) {
      double d0 = 1.0, z = 0.0;
      if (!sign_mode) minmax_params(mn, mx, a.bits, d0, z);
      rp[r * 4 + 0] = d0;
      rp[r * 4 + 1] = z;
      rp[r * 4 + 2] = sabs / (double)beta;
    }
    if (a.omega) {
      for (int c = lane; c < beta; c += 64) om[r * beta + c] = a.omega[(int64_t)(r0 + r) * beta + c];
    } else {
      for (int c = lane; c < beta; c += 64) {
        const double d = a.dblk[c];
        om[r * beta + c] = (w[c] * w[c]) / (d * d);
      }
    }
  }
  __syncthreads();

  // A pair of neighbouring lanes takes SQC_CPT consecutive candidates of one row, each lane half of the row's
  // weights: a weight and its loss weight are read from LDS once for four candidates, the four losses form
  // independent dependency chains, and there are enough wavefronts to hide the latency of the fp64 pipeline.
  const double qmax = (double)((1 << a.bits) - 1);
  const int tpr = (ncand + SQC_CPT - 1) / SQC_CPT;      // lane pairs per row
  const int hb = beta / 2;
  for (int s0 = 0; s0 < 2 * rows * tpr; s0 += SQC_THREADS) {
    const int s = s0 + tid;
    const bool live = s < 2 * rows * tpr;
    const int item = min(s, 2 * rows * tpr - 1) >> 1, half = s & 1;
    const int r = item / tpr, c0 = (item - r * tpr) * SQC_CPT;
    const double* w = wrow + r * beta + half * hb;
    const double* o = om + r * beta + half * hb;
    double L[SQC_CPT], dl[SQC_CPT], rd[SQC_CPT];
#pragma unroll
    for (int i = 0; i < SQC_CPT; ++i) {
      const double tc = a.tau[min(c0 + i, ncand - 1)];
      L[i] = 0.0;
      // SIGN: the level tau * alpha; otherwise the step tau * delta0 and its reciprocal.  The loss is continuous
      // across a rounding tie (both neighbouring codes are equally far), so the candidate losses may use a
      // reciprocal; the codes themselves are decided with a true division.
      dl[i] = tc * (sign_mode ? rp[r * 4 + 2] : rp[r * 4 + 0]);
      rd[i] = 1.0 / dl[i];
    }
    if (sign_mode) {
      for (int j = 0; j < hb; ++j) {
        const double v = w[j], oj = o[j];
#pragma unroll
        for (int i = 0; i < SQC_CPT; ++i) {
          const double e = v - (v >= 0.0 ? dl[i] : -dl[i]);
          L[i] = fma(oj * e, e, L[i]);
        }
      }
    } else {
      // clamp(rint(x) + z, 0, qmax) - z == clamp(rint(x), -z, qmax - z): one add and one subtract less per element
      const double z = rp[r * 4 + 1];
      const double lo = -z, hi = qmax - z;
      for (int j = 0; j < hb; j += 2) {
        const double2 v2 = *reinterpret_cast<const double2*>(w + j);
        const double2 o2 = *reinterpret_cast<const double2*>(o + j);
#pragma unroll
        for (int i = 0; i < SQC_CPT; ++i) {
          const double q0 = fmin(fmax(rint(v2.x * rd[i]), lo), hi);
          const double e0 = fma(-dl[i], q0, v2.x);
          L[i] = fma(o2.x * e0, e0, L[i]);
        }
#pragma unroll
        for (int i = 0; i < SQC_CPT; ++i) {
          const double q1 = fmin(fmax(rint(v2.y * rd[i]), lo), hi);
          const double e1 = fma(-dl[i], q1, v2.y);
          L[i] = fma(o2.y * e1, e1, L[i]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < SQC_CPT; ++i) {
      const double other = shfl_xor_f64(L[i], 1);          // the other half of the row, from the neighbouring lane
      if (live && half == 0 && c0 + i < ncand) loss[r * ncand + c0 + i] = L[i] + other;
    }
  }
  __syncthreads();

  // first minimum per row
  for (int r = wave; r < rows; r += SQC_THREADS / 64) {
    double best = INFINITY;
    int bi = 0x7fffffff;
    for (int c = lane; c < ncand; c += 64) {
      const double L = loss[r * ncand + c];
      if (L < best) {
        best = L;
        bi = c;
      }
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) {
      const double ob = shfl_xor_f64(best, s);
      const int oi = __shfl_xor(bi, s, 64);
      if (ob < best || (ob == best && oi < bi)) {
        best = ob;
        bi = oi;
      }
    }
    if (lane == 0) {
      if (bi == 0x7fffffff) bi = 0;
      const int64_t o = (int64_t)(r0 + r) * a.out_stride;
      const double tc = a.tau[bi];
      if (sign_mode) {
        a.scale[o] = 2.0 * tc * rp[r * 4 + 2];
        a.zero[o] = 0.5;
      } else {
        a.scale[o] = tc * rp[r * 4 + 0];
        a.zero[o] = rp[r * 4 + 1];
      }
      if (a.cand_idx) a.cand_idx[o] = bi;
    }
  }
}

// rows per workgroup: as many as fill the 256 threads with (row, four candidates, half row) items, 16 at most
int sqc_rows_per_wg(int ncand) {
  const int tpr = (ncand + SQC_CPT - 1) / SQC_CPT;
  return std::max(1, std::min(16, SQC_THREADS / (2 * tpr)));
}

size_t sqc_smem_bytes(int beta, int ncand, int rows) {
  return sizeof(double) * ((size_t)2 * rows * beta + (size_t)rows * ncand + rows * 4);
}

// ------------------------------------------------------------------------------------------
// Column sweep of one group: arguments and helpers.
// ------------------------------------------------------------------------------------------
struct SweepArgs {
  double* W;             // working copy, pointer to the block's first column
  int64_t ldw;
  int n, beta, bits, q1_mode;
  const double* U;       // pointer to U[b0][b0]
  int64_t ldu;
  const double* scale;   // element i at scale[i * sz_stride]
  const double* zero;
  int64_t sz_stride;
  uint8_t* codes;        // pointer to codes[0][b0]
  int64_t ldc;
  double* E;             // n x beta block of the error matrix
  int64_t lde;
  double* row_e2;        // n running sums of e^2
  void* What;            // pointer to What[0][b0] or null
  int64_t ldwh;
  int what_f64;
  int sets;              // sets of rows each wavefront sweeps one after the other
};

// fmax / fmin without the canonicalisation of the operands that the compiler would add in front of every use
// (the operands here are never signalling NaNs)
__device__ __forceinline__ double vmax_f64(double a, double b) {
#if defined(__HIP_DEVICE_COMPILE__)
  double r;
  asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
#else
  return a > b ? a : b;
#endif
}
__device__ __forceinline__ double vmin_f64(double a, double b) {
#if defined(__HIP_DEVICE_COMPILE__)
  double r;
  asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
#else
  return a < b ? a : b;
#endif
}

// ------------------------------------------------------------------------------------------
// sqc_search_fast: the candidate search for the two loss weightings that need no weight per element, the default
// L = L_s / |s| + L_us / |us| over the 3-sigma mask and the unweighted Eq. 5.  Both are read off two plain sums
// of squared errors: over all weights of the row (the main loop, six fp64 instructions per weight and candidate:
// multiply by the reciprocal step, round, clamp twice, error, accumulate) and over the few salient ones, which a
// second short loop visits again; L = (all - salient) / |us| + salient / |s|.
// Four neighbouring lanes (a quad) share a (row, 5 candidates) item, each taking every fourth pair of weights,
// so a weight pair read from LDS serves ten loss chains; with 100 candidates a row is 80 threads and a workgroup
// of 320 threads takes four rows, which gives every SIMD of a CU the same number of wavefronts.  Reductions go
// through DPP inside a 16-lane row and lane reads across rows.
// ------------------------------------------------------------------------------------------
typedef double double2v __attribute__((ext_vector_type(2)));
constexpr int SQF_CPT = 5;     // candidates per lane
constexpr int SQF_PAD = 8;     // doubles of padding per LDS row

// reciprocal to full precision without the division sequence (two Newton steps on the hardware estimate)
__device__ __forceinline__ double fast_rcp(double d) {
  double r = __builtin_amdgcn_rcp(d);
  r = fma(fma(-d, r, 1.0), r, r);
  r = fma(fma(-d, r, 1.0), r, r);
  return r;
}

__global__ __launch_bounds__(1024, 5) void sqc_search_fast(SqcArgs a) {
  extern __shared__ __align__(16) double smem[];
  const int beta = a.beta, ncand = a.ncand, RW = a.rows_per_wg;
  const int stride = beta + SQF_PAD;
  double* wrow = smem;                            // [RW][stride]  the rows' weights
  double* sal = wrow + RW * stride;               // [RW][stride]  each row's salient weights, compacted
  double* loss = sal + RW * stride;               // [RW][ncand]
  double* rp = loss + RW * ncand;                 // [RW][8]: delta0, z, alpha, 1/|s|, 1/|us|, |s|, row sum
  double* red = rp + RW * 8;                      // [2 * 16]
  double* tgrid = red + 32;                       // [ncand]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const bool sign_mode = (a.bits == 1 && a.q1_mode == SLIM_Q1_SIGN);
  const bool need_mask = (a.weight_mode == SLIM_WEIGHT_MASK_MEAN);
  const bool block_scope = need_mask && a.scope == SLIM_SCOPE_BLOCK;
  const int nsets = (a.n + RW - 1) / RW;

  // A workgroup takes sets of RW rows in turn.  When a wavefront has one row to fetch and it fits two
  // registers per lane, the rows of the next set are fetched before the search of the current one starts.
  const bool ahead = RW <= nwaves && beta <= 128;
  double pre[2] = {0.0, 0.0};
  auto fetch_row = [&](int set) {
    const int row = set * RW + wave;
    if (set < nsets && wave < RW && row < a.n) {
      const double* src = a.W + (int64_t)row * a.ldw;
#pragma unroll
      for (int q = 0; q < 2; ++q)
        if (q * 64 + lane < beta) pre[q] = src[q * 64 + lane];
    }
  };
  if (ahead) fetch_row(blockIdx.x);

  // the candidate grid goes to LDS once
  for (int c = tid; c < ncand; c += blockDim.x) tgrid[c] = a.tau[c];
  const int groups = (ncand + SQF_CPT - 1) / SQF_CPT;
  const int tpr = 4 * groups;
  // block-wide mean and 3 sigma from the slab partials, once per workgroup, summed in a fixed order
  double mu = 0.0, thr = 0.0;
  if (block_scope) {
    double s1 = 0.0, s2 = 0.0;
    for (int p = tid; p < a.nstat; p += blockDim.x) {
      s1 += a.stat_partial[2 * p];
      s2 += a.stat_partial[2 * p + 1];
    }
    s1 = wave_allreduce<OpSum>(s1);
    s2 = wave_allreduce<OpSum>(s2);
    if (lane == 0) {
      red[2 * wave] = s1;
      red[2 * wave + 1] = s2;
    }
    __syncthreads();
    double S1 = 0.0, S2 = 0.0;
    for (int w = 0; w < nwaves; ++w) {
      S1 += red[2 * w];
      S2 += red[2 * w + 1];
    }
    const double cnt = (double)a.n * (double)beta;
    const double m1 = S1 / cnt;
    const double var = fmax(S2 / cnt - m1 * m1, 0.0);
    mu = a.W[0] + m1;
    thr = 3.0 * sqrt(var);
  }
  const double qmax = (double)((1 << a.bits) - 1);

  for (int set = blockIdx.x; set < nsets; set += gridDim.x) {
    const int r0 = set * RW;
    const int rows = min(RW, a.n - r0);
    // a wavefront per row: the row goes to LDS; its minimum, maximum and sum of magnitudes give the parameters,
    // its salient weights are copied to the row's list and their number decides the two loss weights
    for (int r = wave; r < rows; r += nwaves) {
      const double* src = a.W + (int64_t)(r0 + r) * a.ldw;
      double* w = wrow + r * stride;
      double mn = INFINITY, mx = -INFINITY, sabs = 0.0, sum = 0.0;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int c = q * 64 + lane;
        if (c < beta) {
          const double v = ahead ? pre[q] : src[c];
          w[c] = v;
          mn = fmin(mn, v);
          mx = fmax(mx, v);
          sabs += fabs(v);
          sum += v;
        }
      }
      for (int c = 128 + lane; c < beta; c += 64) {
        const double v = src[c];
        w[c] = v;
        mn = fmin(mn, v);
        mx = fmax(mx, v);
        sabs += fabs(v);
        sum += v;
      }
      mn = wave_allreduce<OpMin>(mn);
      mx = wave_allreduce<OpMax>(mx);
      sabs = wave_allreduce<OpSum>(sabs);
      int ns = 0;
      if (need_mask) {
        double rmu = mu, rthr = thr;
        if (!block_scope) {
          rmu = wave_allreduce<OpSum>(sum) / (double)beta;
          double ss = 0.0;
          for (int c = lane; c < beta; c += 64) {
            const double d = w[c] - rmu;
            ss += d * d;
          }
          ss = wave_allreduce<OpSum>(ss);
          rthr = 3.0 * sqrt(ss / (double)beta);
        }
        for (int c0 = 0; c0 < beta; c0 += 64) {
          const int c = c0 + lane;
          const double v = c < beta ? w[c] : 0.0;
          const bool s = c < beta && fabs(v - rmu) > rthr;
          const unsigned long long b = __ballot(s);
          const int before = __builtin_amdgcn_mbcnt_hi((unsigned)(b >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)b, 0u));
          if (s) sal[r * stride + ns + before] = v;
          ns += __builtin_popcountll(b);
        }
      }
      if (lane == 0) {
        double d0 = 1.0, z = 0.0;
        if (!sign_mode) minmax_params(mn, mx, a.bits, d0, z);
        const int nus = beta - ns;
        double ws = 0.0, wus = 1.0;
        if (need_mask) {
          ws = ns ? fast_rcp((double)ns) : 0.0;
          wus = nus ? fast_rcp((double)nus) : 0.0;
        }
        rp[r * 8 + 0] = d0;
        rp[r * 8 + 1] = z;
        rp[r * 8 + 2] = sabs / (double)beta;
        rp[r * 8 + 3] = ws;
        rp[r * 8 + 4] = wus;
        reinterpret_cast<int*>(rp + r * 8 + 5)[0] = ns;
      }
    }
    if (ahead) fetch_row(set + gridDim.x);
    __syncthreads();

    // main loop: a quad of lanes per (row, SQF_CPT candidates)
    for (int s0 = 0; s0 < rows * tpr; s0 += blockDim.x) {
      const int s = s0 + tid;
      const bool live = s < rows * tpr;
      const int sc = min(s, rows * tpr - 1);
      const int r = sc / tpr, rem = sc - r * tpr;
      const int c0 = (rem >> 2) * SQF_CPT, p = rem & 3;
      const double* w = wrow + r * stride;
      const double* sl = sal + r * stride;
      const double* par = rp + r * 8;
      const int ns = reinterpret_cast<const int*>(par + 5)[0];
      // L = wus * (sum over all) + (ws - wus) * (sum over the salient ones)
      const double wus = par[4], wdiff = par[3] - par[4];
      double L[SQF_CPT], dl[SQF_CPT], rd[SQF_CPT];
#pragma unroll
      for (int i = 0; i < SQF_CPT; ++i) {
        const double tc = tgrid[min(c0 + i, ncand - 1)];
        L[i] = 0.0;
        // SIGN: the level tau * alpha; otherwise the step tau * delta0 and its reciprocal.  The loss is continuous
        // across a rounding tie (both neighbouring codes are equally far), so the candidate losses may use a
        // reciprocal; the codes themselves are decided with a true division.
        dl[i] = tc * (sign_mode ? par[2] : par[0]);
        rd[i] = fast_rcp(dl[i]);
      }
      if (sign_mode) {
        // |w - sign(w) level| = ||w| - level|
        for (int j = 0; j < beta / 8; ++j) {
          const double2v v2 = *reinterpret_cast<const double2v*>(w + (4 * j + p) * 2);
#pragma unroll
          for (int i = 0; i < SQF_CPT; ++i) {
            const double e0 = fabs(v2.x) - dl[i], e1 = fabs(v2.y) - dl[i];
            L[i] = fma(e0, e0, L[i]);
            L[i] = fma(e1, e1, L[i]);
          }
        }
#pragma unroll
        for (int i = 0; i < SQF_CPT; ++i) L[i] *= wus;
        for (int j = p; j < ns; j += 4) {
          const double v = sl[j];
#pragma unroll
          for (int i = 0; i < SQF_CPT; ++i) {
            const double e = fabs(v) - dl[i];
            L[i] = fma(e * wdiff, e, L[i]);
          }
        }
      } else {
        // clamp(rint(x) + z, 0, qmax) - z == clamp(rint(x), -z, qmax - z): one add and one subtract less per element
        const double z = par[1];
        const double lo = -z, hi = qmax - z;
        double2v nxt = *reinterpret_cast<const double2v*>(w + p * 2);
        for (int j = 0; j < beta / 8; ++j) {
          const double2v v2 = nxt;
          nxt = *reinterpret_cast<const double2v*>(w + (4 * min(j + 1, beta / 8 - 1) + p) * 2);   // one pair ahead
          // stage by stage over the five candidates' independent chains, so that a wavefront need not wait on
          // its own results
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const double v = h ? v2.y : v2.x;
            double x[SQF_CPT];
#pragma unroll
            for (int i = 0; i < SQF_CPT; ++i) x[i] = v * rd[i];
#pragma unroll
            for (int i = 0; i < SQF_CPT; ++i) x[i] = rint(x[i]);
#pragma unroll
            for (int i = 0; i < SQF_CPT; ++i) x[i] = fmax(x[i], lo);
#pragma unroll
            for (int i = 0; i < SQF_CPT; ++i) x[i] = fmin(x[i], hi);
#pragma unroll
            for (int i = 0; i < SQF_CPT; ++i) x[i] = fma(-dl[i], x[i], v);
#pragma unroll
            for (int i = 0; i < SQF_CPT; ++i) L[i] = fma(x[i], x[i], L[i]);
          }
        }
#pragma unroll
        for (int i = 0; i < SQF_CPT; ++i) L[i] *= wus;
        for (int j = p; j < ns; j += 4) {
          const double v = sl[j];
#pragma unroll
          for (int i = 0; i < SQF_CPT; ++i) {
            const double q = fmin(fmax(rint(v * rd[i]), lo), hi);
            const double e = fma(-dl[i], q, v);
            L[i] = fma(e * wdiff, e, L[i]);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < SQF_CPT; ++i) {
        double t = L[i];                                   // this lane's share: the loss is linear in the sums
        t += dpp_f64<DPP_XOR1>(t);
        t += dpp_f64<DPP_XOR2>(t);
        if (live && p == 0 && c0 + i < ncand) loss[r * ncand + c0 + i] = t;
      }
    }
    __syncthreads();

    // first minimum per row
    for (int r = wave; r < rows; r += nwaves) {
      double best = INFINITY;
      int bi = 0x7fffffff;
      for (int c = lane; c < ncand; c += 64) {
        const double L = loss[r * ncand + c];
        if (L < best) {
          best = L;
          bi = c;
        }
      }
#define SQF_ARGMIN_STEP(CTRL)                                                   \
      {                                                                           \
        const double ob = dpp_f64<CTRL>(best);                                    \
        const int oi = dpp_b32<CTRL>(bi);                                         \
        if (ob < best || (ob == best && oi < bi)) {                               \
          best = ob;                                                              \
          bi = oi;                                                                \
        }                                                                         \
      }
      SQF_ARGMIN_STEP(DPP_XOR1)
      SQF_ARGMIN_STEP(DPP_XOR2)
      SQF_ARGMIN_STEP(DPP_HALF_MIRROR)
      SQF_ARGMIN_STEP(DPP_MIRROR)
#undef SQF_ARGMIN_STEP
#pragma unroll
      for (int src = 16; src < 64; src += 16) {
        const double ob = read_lane_f64(best, src);
        const int oi = __builtin_amdgcn_readlane(bi, src);
        if (lane == 0 && (ob < best || (ob == best && oi < bi))) {
          best = ob;
          bi = oi;
        }
      }
      if (lane == 0) {
        if (bi == 0x7fffffff) bi = 0;
        const int64_t o = (int64_t)(r0 + r) * a.out_stride;
        const double tc = tgrid[bi];
        if (sign_mode) {
          a.scale[o] = 2.0 * tc * rp[r * 8 + 2];
          a.zero[o] = 0.5;
        } else {
          a.scale[o] = tc * rp[r * 8 + 0];
          a.zero[o] = rp[r * 8 + 1];
        }
        if (a.cand_idx) a.cand_idx[o] = bi;
      }
    }
  }
}

// launch shape of sqc_search_fast: rows per workgroup and threads
void sqf_shape(int beta, int ncand, int& rows, int& threads, size_t& smem) {
  const int tpr = 4 * ((ncand + SQF_CPT - 1) / SQF_CPT);
  rows = std::max(1, std::min(16, 320 / tpr));
  const size_t per_row = sizeof(double) * (2 * (size_t)(beta + SQF_PAD) + ncand + 8);
  rows = (int)std::max<size_t>(1, std::min<size_t>(rows, (60 * 1024) / per_row));
  threads = std::min(1024, ((rows * tpr + 63) / 64) * 64);
  smem = rows * per_row + sizeof(double) * (32 + ncand);
}

// ------------------------------------------------------------------------------------------
// The sweep itself, four rows per wavefront.  Most instructions of a step work on values that are the same for
// every lane of a row (the current weight, its code, the error), so a wavefront that carried one row would
// spend 64 lanes on them.  Here a row takes 16 lanes (one DPP row): lane l of a row holds columns
// l, l + 16, ... of the group, v_mov_b32_dpp row_newbcast hands the current column to the 16 lanes of each row,
// and the scalar work of a step serves four rows at once.  The steps are unrolled completely (the DPP lane is
// an immediate), so every LDS offset is a constant.  Row j of the U block keeps only the columns from the start
// of its 16-column segment on, which halves the block in LDS.
// ------------------------------------------------------------------------------------------
constexpr int SWEEP4_RPW = 4;   // rows per wavefront

// offset of row 16 k + jj of the packed U block (rows of segment k' hold BETA - 16 k' entries)
__host__ __device__ constexpr int sweep4_row_off(int beta, int k, int jj) {
  return 16 * k * beta - 128 * k * (k - 1) + jj * (beta - 16 * k);
}

template <int N>
__device__ __forceinline__ double bcast_row16(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, 0x150 + N, 0xf, 0xf, true);   // row_newbcast:N, every lane written
  hi = __builtin_amdgcn_update_dpp(0, hi, 0x150 + N, 0xf, 0xf, true);
  return __hiloint2double(hi, lo);
}

template <int BETA>
struct Sweep4 {
  static constexpr int NK = BETA / 16;
  double w[NK];          // the row's weights: w[k] is column 16 k + l16
  double u[NK];          // row j of U / U_jj for the current step (entries k >= j / 16)
  double wj;             // the current column's weight, the same in the row's 16 lanes
  double rd;             // 1 / U_jj
  double ujn;            // U_{j,j+1} / U_jj
  double s, rs, z, lo, hi, e2;
  const double* Ub;      // packed, row-scaled U block
  const double* rdiag;
  // Index bases kept in registers (opaque to the compiler), so that every LDS read of the unrolled steps is one of
  // these plus an immediate offset below 64 KiB: 0 and HI for the reads that are the same in every lane, l16 and
  // l16 + HI for a lane's own columns.
  static constexpr int HI = 4096;
  int u0, uh, l0, lh;
  template <int OFF> __device__ __forceinline__ double uni() const {
    return OFF < HI ? Ub[u0 + OFF] : Ub[uh + (OFF - HI)];
  }
  // index of entry OFF of the packed block plus the lane's own column offset
  template <int OFF> __device__ __forceinline__ int mine() const { return OFF < HI ? l0 + OFF : lh + (OFF - HI); }
  double* eb;            // this row's beta errors
  uint8_t* qb;           // this row's beta codes
};

// One step.  A lone wavefront per SIMD is bound by the chain of dependent fp64 instructions from one column's
// weight to the next one's (each costs some 32 cycles), so the chain is kept to
//   w_j -> * 1/s -> round -> max -> min -> d = w_j - s (q - z) -> w_{j+1} = bcast(w[j+1]) - d U'_{j,j+1}:
// the rows of U are stored divided by their diagonal element (U' = U / U_jj, so the update is w -= d U' and the
// error e = d / U_jj is formed beside the chain), the next column's weight is updated by itself from a broadcast
// taken before this step's update, and the tie check is evaluated beside the clamp and acted on afterwards.
template <int BETA, bool SIGN, int K, int JJ>
__device__ __forceinline__ void sweep4_step(Sweep4<BETA>& st) {
  constexpr int NK = BETA / 16, J = 16 * K + JJ;
  constexpr int K1 = (J + 1) / 16, JJ1 = (J + 1) % 16;
  // the next step's row of U' and reciprocal, fetched ahead of this step's arithmetic
  double un[NK];
  double rdn = 0.0, ujnn = 0.0, wpre = 0.0;
  if constexpr (J + 1 < BETA) {
    constexpr int off = sweep4_row_off(BETA, K1, JJ1);
#pragma unroll
    for (int k2 = K1; k2 < NK; ++k2) un[k2] = st.Ub[st.template mine<off>() + (k2 - K1) * 16];
    rdn = st.rdiag[st.u0 + J + 1];
    if constexpr (J + 2 < BETA) ujnn = st.template uni<off + JJ1 + 1>();   // U'_{j+1,j+2}
    wpre = bcast_row16<JJ1>(st.w[K1]);                         // w_{j+1} before this step's update
  }
  const double wj = st.wj;
  double qz, d;                                // q - z and w_j - s (q - z)
  if (SIGN) {
    qz = (wj >= 0.0) ? 0.5 : -0.5;
    d = fma(-st.s, qz, wj);
  } else {
    // The code is rint(wj / s) with a true division.  wj * (1 / s) lies within a few ulps of the quotient, so
    // unless it is that close to a rounding tie it rounds the same way; only then (practically never) is the
    // division done (a real branch: the asm keeps the compiler from computing the quotient speculatively).
    // Codes are clamped to a few units around zero, so 1e-7 is far above a few ulps of any x that matters.
    const double x = wj * st.rs;
    const double xr = rint(x);
    qz = vmin_f64(vmax_f64(xr, st.lo), st.hi);
    d = fma(-st.s, qz, wj);
    if (fabs(x - xr) > 0.5 - 1e-7) {
      double xd = wj / st.s;
      asm volatile("" : "+v"(xd));
      qz = vmin_f64(vmax_f64(rint(xd), st.lo), st.hi);
      d = fma(-st.s, qz, wj);
    }
  }
  if constexpr (J + 1 < BETA) st.wj = fma(-d, st.ujn, wpre);
#pragma unroll
  for (int k2 = K; k2 < NK; ++k2) {
    st.w[k2] = fma(-d, st.u[k2], st.w[k2]);
    // Later segments' weights are not read for many steps; without this the compiler sinks their updates down to
    // the first use and keeps every step's d and row of U alive (in scratch) until then.
    asm volatile("" : "+v"(st.w[k2]));
  }
  const double e = d * st.rd;
  st.e2 = fma(e, e, st.e2);
  asm volatile("" : "+v"(st.e2));              // same: keep the running sum here, not every error until the end
  st.eb[J] = e;
  st.qb[J] = (uint8_t)(int)(qz + st.z);
  if constexpr (J + 1 < BETA) {
#pragma unroll
    for (int k2 = K1; k2 < NK; ++k2) st.u[k2] = un[k2];
    st.rd = rdn;
    st.ujn = ujnn;
  }
  // The steps are one long straight line; left alone, the scheduler hoists the LDS reads of many steps to the
  // top and runs out of registers.
  __builtin_amdgcn_sched_barrier(0);
}

template <int BETA, bool SIGN, int K, int... JJ>
__device__ __forceinline__ void sweep4_segment(Sweep4<BETA>& st, std::integer_sequence<int, JJ...>) {
  (sweep4_step<BETA, SIGN, K, JJ>(st), ...);
}
template <int BETA, bool SIGN, int... K>
__device__ __forceinline__ void sweep4_all(Sweep4<BETA>& st, std::integer_sequence<int, K...>) {
  (sweep4_segment<BETA, SIGN, K>(st, std::make_integer_sequence<int, 16>{}), ...);
}

// LDS of gptq_sweep4: packed U block, reciprocals of its diagonal, then per row BETA errors and BETA codes
size_t sweep4_smem_bytes(int beta, int waves) {
  const int rows = waves * SWEEP4_RPW;
  const size_t packed = (size_t)sweep4_row_off(beta, beta / 16, 0);
  return sizeof(double) * (packed + beta + (size_t)rows * beta) + (size_t)rows * beta;
}

template <int BETA, bool SIGN>
__global__ __launch_bounds__(1024) void gptq_sweep4(SweepArgs a) {
  constexpr int NK = BETA / 16, PACKED = sweep4_row_off(BETA, NK, 0);
  extern __shared__ __align__(16) double Us[];
  const int tid = threadIdx.x, nthreads = blockDim.x, lane = tid & 63, wave = tid >> 6;
  const int rows_per_wg = (nthreads >> 6) * SWEEP4_RPW;
  double* rdiag = Us + PACKED;
  double* ebase = rdiag + BETA;
  uint8_t* qbase = reinterpret_cast<uint8_t*>(ebase + rows_per_wg * BETA);
  for (int j = tid; j < BETA; j += nthreads) rdiag[j] = 1.0 / a.U[(int64_t)j * a.ldu + j];
  __syncthreads();
  // The packed block, two columns at a time: only the upper triangle is meaningful, and each row is divided by
  // its diagonal element.  Six loads are in flight per thread before the first is used (the block comes from L2,
  // and with few wavefronts per workgroup the fill would otherwise be a string of round trips).
  constexpr int FILL = 6;
  for (int i0 = tid; i0 < PACKED / 2; i0 += FILL * nthreads) {
    double2 v[FILL];
    int jrow[FILL], col[FILL];
#pragma unroll
    for (int q = 0; q < FILL; ++q) {
      const int e = 2 * (i0 + q * nthreads);       // index in the packed block
      v[q] = make_double2(0.0, 0.0);
      if (e < PACKED) {
        int k = 0;
#pragma unroll
        for (int kk = 1; kk < NK; ++kk) k += (e >= sweep4_row_off(BETA, kk, 0)) ? 1 : 0;
        const int width = BETA - 16 * k, r = e - sweep4_row_off(BETA, k, 0);
        const int jj = r / width;
        jrow[q] = 16 * k + jj;
        col[q] = r - jj * width;                   // column within the segment's range, even
        v[q] = *reinterpret_cast<const double2*>(a.U + (int64_t)jrow[q] * a.ldu + 16 * k + col[q]);
      }
    }
#pragma unroll
    for (int q = 0; q < FILL; ++q) {
      const int e = 2 * (i0 + q * nthreads);
      if (e < PACKED) {
        const double rd = rdiag[jrow[q]];
        const int jj = jrow[q] & 15;
        double2 o;
        o.x = (col[q] >= jj) ? v[q].x * rd : 0.0;
        o.y = (col[q] + 1 >= jj) ? v[q].y * rd : 0.0;
        *reinterpret_cast<double2*>(Us + e) = o;
      }
    }
  }
  __syncthreads();

  // No barrier below.  With more rows than one round of workgroups holds, a wavefront sweeps several sets of rows
  // in turn and the workgroup's copy of the U block serves them all.
  const int g = lane >> 4, l16 = lane & 15;
  const int rl = wave * SWEEP4_RPW + g;            // row within the workgroup's current set
  for (int set = 0; set < a.sets; ++set) {
    const int row0 = (blockIdx.x * a.sets + set) * rows_per_wg;
    const int row = row0 + rl;
    if (row0 + wave * SWEEP4_RPW >= a.n) break;
    const bool valid = row < a.n;                    // rows past the end compute on zeros and store nothing

    Sweep4<BETA> st;
    const double qmax = (double)((1 << a.bits) - 1);
    st.s = valid ? a.scale[(int64_t)row * a.sz_stride] : 1.0;
    st.z = valid ? a.zero[(int64_t)row * a.sz_stride] : 0.0;
    st.rs = 1.0 / st.s;
    st.lo = -st.z;                                   // clamp(rint(x) + z, 0, qmax) - z == clamp(rint(x), lo, hi)
    st.hi = qmax - st.z;
    st.e2 = 0.0;
    st.Ub = Us;
    st.rdiag = rdiag;
    st.u0 = 0;
    st.uh = Sweep4<BETA>::HI;
    st.l0 = l16;
    st.lh = l16 + Sweep4<BETA>::HI;
    asm volatile("" : "+v"(st.u0), "+v"(st.uh), "+v"(st.l0), "+v"(st.lh));
    st.eb = ebase + rl * BETA;
    st.qb = qbase + rl * BETA;
    const double* wr = a.W + (int64_t)row * a.ldw;
#pragma unroll
    for (int k = 0; k < NK; ++k) st.w[k] = valid ? wr[16 * k + l16] : 0.0;
#pragma unroll
    for (int k = 0; k < NK; ++k) st.u[k] = Us[l16 + 16 * k];
    st.rd = rdiag[0];
    st.ujn = Us[1];
    st.wj = bcast_row16<0>(st.w[0]);
    asm volatile("" : "+v"(st.lo));                  // opaque, or -z is formed again in every step
    sweep4_all<BETA, SIGN>(st, std::make_integer_sequence<int, NK>{});

    // each lane picks up the errors and codes of its own columns (written by its own wavefront)
    if (valid) {
#pragma unroll
      for (int k = 0; k < NK; ++k) {
        const int c = 16 * k + l16;
        const double ev = st.eb[c];
        const uint8_t code = st.qb[c];
        a.codes[(int64_t)row * a.ldc + c] = code;
        a.E[(int64_t)row * a.lde + c] = ev;
        if (a.What) {
          const double what = st.s * ((double)code - st.z);
          if (a.what_f64)
            static_cast<double*>(a.What)[(int64_t)row * a.ldwh + c] = what;
          else
            static_cast<float*>(a.What)[(int64_t)row * a.ldwh + c] = (float)what;
        }
      }
      if (l16 == 0) a.row_e2[row] += st.e2;
    }
  }
}

// Kernels that may need more than the default 64 KiB of dynamic LDS opt in once per process.
template <typename K>
slim_status allow_big_lds(slim_ctx* ctx, K kernel, bool& done) {
  if (!done) {
    SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    done = true;
  }
  return SLIM_OK;
}

bool beta_supported(int beta) { return beta == 32 || beta == 64 || beta == 128 || beta == 256 || beta == 512; }

slim_status launch_stats_and_sqc(slim_ctx* ctx, SqcArgs a, double* stat_partial) {
  const bool need_block_stats =
      (a.omega == nullptr && a.weight_mode == SLIM_WEIGHT_MASK_MEAN && a.scope == SLIM_SCOPE_BLOCK);
  a.stat_partial = nullptr;
  a.nstat = 0;
  if (need_block_stats) {
    a.nstat = slim_cdiv(a.n, STAT_ROWS);
    a.stat_partial = stat_partial;
    SLIM_LAUNCH(ctx, "sqc_block_stats", block_stats, dim3(a.nstat), dim3(256), 0, a.W, a.ldw, a.n, a.beta, stat_partial);
  }
  if (a.omega == nullptr && (a.weight_mode == SLIM_WEIGHT_MASK_MEAN || a.weight_mode == SLIM_WEIGHT_UNIFORM)) {
    int threads = 0;
    size_t smem = 0;
    sqf_shape(a.beta, a.ncand, a.rows_per_wg, threads, smem);
    if (smem > 64 * 1024) {
      static bool done = false;
      slim_status st = allow_big_lds(ctx, sqc_search_fast, done);
      if (st != SLIM_OK) return st;
    }
    // no more workgroups than are resident at once: each takes sets of rows in turn and fetches ahead
    int per_cu = 0;
    SLIM_HIP_TRY(ctx, hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sqc_search_fast, threads, smem));
    const int wgs = std::min(slim_cdiv(a.n, a.rows_per_wg), std::max(1, per_cu) * std::max(1, ctx->num_cus));
    SLIM_LAUNCH(ctx, "sqc_search", sqc_search_fast, dim3(wgs), dim3(threads), smem, a);
    return SLIM_OK;
  }
  a.rows_per_wg = sqc_rows_per_wg(a.ncand);
  const size_t smem = sqc_smem_bytes(a.beta, a.ncand, a.rows_per_wg);
  if (smem > 160 * 1024) return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "sqc: beta * ncand too large for LDS");
  if (smem > 64 * 1024) {
    static bool done = false;
    slim_status st = allow_big_lds(ctx, sqc_search_weighted, done);
    if (st != SLIM_OK) return st;
  }
  SLIM_LAUNCH(ctx, "sqc_search", sqc_search_weighted, dim3(slim_cdiv(a.n, a.rows_per_wg)), dim3(SQC_THREADS), smem, a);
  return SLIM_OK;
}

slim_status check_params(slim_ctx* ctx, const slim_params* p, slim_params& out) {
  slim_default_params(&out);
  if (p) out = *p;
  SLIM_REQUIRE(ctx, out.sqc_weight_mode >= 0 && out.sqc_weight_mode <= 2, "unknown sqc_weight_mode %d", out.sqc_weight_mode);
  SLIM_REQUIRE(ctx, out.mask_scope == 0 || out.mask_scope == 1, "unknown mask_scope %d", out.mask_scope);
  SLIM_REQUIRE(ctx, out.q1_mode == 0 || out.q1_mode == 1, "unknown q1_mode %d", out.q1_mode);
  SLIM_REQUIRE(ctx, out.sal_mode == 0 || out.sal_mode == 1, "unknown sal_mode %d", out.sal_mode);
  return SLIM_OK;
}

}  // namespace

size_t slim_ws_need_sqc(int n) { return slim_ws_round(sizeof(double) * 2 * slim_cdiv(n, STAT_ROWS)); }

size_t slim_ws_need_gptq(int n, int m) {
  return slim_ws_round(sizeof(double) * (size_t)n * m) + slim_ws_round(sizeof(double) * (size_t)n * GPTQ_WINC) +
         slim_ws_round(sizeof(double) * 2 * slim_cdiv(n, STAT_ROWS)) + slim_ws_round(sizeof(double) * n);
}

extern "C" slim_status slim_sqc_calibrate(slim_ctx* ctx, const double* Wblk, int64_t ldw, int n, int beta, int bits,
                                          const double* omega, const double* hinv_diag_blk,
                                          const slim_params* params, const double* tau, int ncand, double* scale,
                                          double* zero, int* cand_idx) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  slim_params prm;
  slim_status st = check_params(ctx, params, prm);
  if (st != SLIM_OK) return st;
  SLIM_REQUIRE(ctx, Wblk && scale && zero, "slim_sqc_calibrate: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && ldw >= beta, "slim_sqc_calibrate: need n > 0 and ldw >= beta");
  SLIM_REQUIRE(ctx, bits >= 1 && bits <= 8, "slim_sqc_calibrate: bits must be in 1..8 (got %d)", bits);
  if (!beta_supported(beta))
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_sqc_calibrate: beta must be 32, 64, 128, 256 or 512 (got %d)", beta);
  if (!tau) {
    tau = ctx->tau_default;
    ncand = ctx->ncand_default;
  }
  SLIM_REQUIRE(ctx, ncand >= 1 && ncand <= SLIM_MAX_CAND, "slim_sqc_calibrate: ncand must be in 1..%d", SLIM_MAX_CAND);
  SLIM_REQUIRE(ctx, !(omega == nullptr && prm.sqc_weight_mode == SLIM_WEIGHT_ELEMENT && hinv_diag_blk == nullptr),
               "slim_sqc_calibrate: ELEMENT weights need hinv_diag_blk");
  const int nstat = slim_cdiv(n, STAT_ROWS);
  st = slim_ws_reserve(ctx, slim_ws_need_sqc(n));
  if (st != SLIM_OK) return st;
  double* stat_partial = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * 2 * nstat));
  SqcArgs a;
  a.W = Wblk;
  a.ldw = ldw;
  a.n = n;
  a.beta = beta;
  a.bits = bits;
  a.omega = omega;
  a.dblk = hinv_diag_blk;
  a.weight_mode = prm.sqc_weight_mode;
  a.scope = prm.mask_scope;
  a.q1_mode = prm.q1_mode;
  a.tau = tau;
  a.ncand = ncand;
  a.scale = scale;
  a.zero = zero;
  a.out_stride = 1;
  a.cand_idx = cand_idx;
  return launch_stats_and_sqc(ctx, a, stat_partial);
}

extern "C" slim_status slim_gptq_quantize(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                                          const double* U, int64_t ldu, const uint8_t* bits, int beta,
                                          int gptq_block, const slim_params* params, const double* hinv_diag,
                                          const double* tau, int ncand, uint8_t* codes, double* scale, double* zero,
                                          void* What, slim_dtype what_dtype, double* sum_e2) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  slim_params prm;
  slim_status st = check_params(ctx, params, prm);
  if (st != SLIM_OK) return st;
  SLIM_REQUIRE(ctx, W && U && bits && codes && scale && zero, "slim_gptq_quantize: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "slim_gptq_quantize: need n, m > 0 and beta | m");
  SLIM_REQUIRE(ctx, ldw >= m && ldw % 4 == 0 && ldu >= m && ldu % 2 == 0, "slim_gptq_quantize: bad leading dimension");
  SLIM_REQUIRE(ctx, slim_aligned16(W) && slim_aligned16(U), "slim_gptq_quantize: misaligned pointer");
  if (!beta_supported(beta))
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_gptq_quantize: beta must be 32, 64, 128, 256 or 512 (got %d)", beta);
  // The sweep works on blocks of at most 128 columns (the beta x beta block of U has to fit in LDS); wider
  // groups are swept in 128-column blocks with a trailing update between them, which gives the same result.
  const int SB = std::min(beta, 128);
  if (gptq_block != beta && gptq_block != SB)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_gptq_quantize: gptq_block must be beta%s", beta > 128 ? " or 128" : "");
  if (w_dtype != SLIM_F16 && w_dtype != SLIM_BF16 && w_dtype != SLIM_F32)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_gptq_quantize: W must be F16, BF16 or F32");
  if (What && what_dtype != SLIM_F32 && what_dtype != SLIM_F64)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_gptq_quantize: What must be F32 or F64");
  if (!tau) {
    tau = ctx->tau_default;
    ncand = ctx->ncand_default;
  }
  SLIM_REQUIRE(ctx, ncand >= 1 && ncand <= SLIM_MAX_CAND, "slim_gptq_quantize: ncand must be in 1..%d", SLIM_MAX_CAND);
  SLIM_REQUIRE(ctx, !(prm.sqc_weight_mode == SLIM_WEIGHT_ELEMENT && hinv_diag == nullptr),
               "slim_gptq_quantize: ELEMENT weights need hinv_diag");
  const int k = m / beta;
  SLIM_REQUIRE(ctx, k <= SLIM_HPIN_BYTES, "slim_gptq_quantize: too many groups");

  // widths to the host: they select kernel arguments, and they must be valid before any output is touched.  The
  // copy is on its way while the working copy of W is made (workspace only), so the stream does not idle for it.
  uint8_t* bits_h = reinterpret_cast<uint8_t*>(ctx->hpin);
  st = slim_ensure_side(ctx);
  if (st != SLIM_OK) return st;
  hipEvent_t ev_bits = ctx->ev[12];
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(bits_h, bits, k, hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipEventRecord(ev_bits, ctx->stream));

  const int nstat = slim_cdiv(n, STAT_ROWS);
  // Trailing updates (Alg. 1 line 12) in two levels: inside a window of WINC columns every swept block updates
  // the rest of the window at once (rank SB); the columns behind the window receive the whole window's errors in
  // one rank-WINC update when its last block is done.  A rank-128 update of everything behind each block moves
  // 16 bytes of W per 32 flops and is bound by memory; this way most of the work has four times that intensity.
  // WINC is a multiple of every supported group size, so a group never straddles a window and the calibration at
  // a group's first column sees columns that have received every earlier block's update.
  constexpr int WINC = GPTQ_WINC;
  st = slim_ws_reserve(ctx, slim_ws_need_gptq(n, m));
  if (st != SLIM_OK) return st;
  double* Wc = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)n * m));
  double* E = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)n * WINC));
  double* stat_partial = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * 2 * nstat));
  double* row_e2 = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * n));

  st = slim_widen_f64(ctx, "gptq_widen", W, w_dtype, n, m, ldw, Wc, (int64_t)m);
  if (st != SLIM_OK) return st;
  st = slim_zero_f64(ctx, "gptq_zero", row_e2, n);
  if (st != SLIM_OK) return st;
  SLIM_HIP_TRY(ctx, hipEventSynchronize(ev_bits));
  std::vector<int> gb(k);
  for (int g = 0; g < k; ++g) {
    gb[g] = bits_h[g];
    SLIM_REQUIRE(ctx, gb[g] >= 1 && gb[g] <= 8, "slim_gptq_quantize: bits[%d] = %d is outside 1..8", g, gb[g]);
  }

  // Rows per workgroup of the sweep: as few as fill the chip, so that small layers spread over every compute
  // unit and large ones share each workgroup's copy of the U block among more rows.
  int sweep_waves = 4;
  while (sweep_waves < 16 && slim_cdiv(n, sweep_waves * SWEEP4_RPW) > ctx->num_cus) sweep_waves *= 2;
  const int sweep_rows = sweep_waves * SWEEP4_RPW;
  const int sweep_sets = std::min(8, slim_cdiv(n, sweep_rows * ctx->num_cus));
  const size_t sweep_smem = sweep4_smem_bytes(SB, sweep_waves);
  if (sweep_smem > 64 * 1024) {
    static bool done0 = false, done1 = false;
    st = allow_big_lds(ctx, gptq_sweep4<128, false>, done0);
    if (st != SLIM_OK) return st;
    st = allow_big_lds(ctx, gptq_sweep4<128, true>, done1);
    if (st != SLIM_OK) return st;
  }

  for (int sb = 0; sb < m / SB; ++sb) {
    const int b0 = sb * SB;
    const int g = b0 / beta;
    const int w0 = (b0 / WINC) * WINC, w1 = std::min(m, w0 + WINC);   // the window of this block
    if (b0 % beta == 0) {
      SqcArgs a;
      a.W = Wc + b0;
      a.ldw = m;
      a.n = n;
      a.beta = beta;
      a.bits = gb[g];
      a.omega = nullptr;
      a.dblk = hinv_diag ? hinv_diag + b0 : nullptr;
      a.weight_mode = prm.sqc_weight_mode;
      a.scope = prm.mask_scope;
      a.q1_mode = prm.q1_mode;
      a.tau = tau;
      a.ncand = ncand;
      a.scale = scale + g;
      a.zero = zero + g;
      a.out_stride = k;
      a.cand_idx = nullptr;
      st = launch_stats_and_sqc(ctx, a, stat_partial);
      if (st != SLIM_OK) return st;
    }

    SweepArgs s;
    s.W = Wc + b0;
    s.ldw = m;
    s.n = n;
    s.beta = SB;
    s.bits = gb[g];
    s.q1_mode = prm.q1_mode;
    s.U = U + (int64_t)b0 * ldu + b0;
    s.ldu = ldu;
    s.scale = scale + g;
    s.zero = zero + g;
    s.sz_stride = k;
    s.codes = codes + b0;
    s.ldc = m;
    s.E = E + (b0 - w0);
    s.lde = WINC;
    s.row_e2 = row_e2;
    s.What = nullptr;
    s.ldwh = m;
    s.what_f64 = (what_dtype == SLIM_F64);
    if (What) {
      s.What = s.what_f64 ? static_cast<void*>(static_cast<double*>(What) + b0)
                          : static_cast<void*>(static_cast<float*>(What) + b0);
    }
    s.sets = sweep_sets;
    const dim3 sgrid(slim_cdiv(n, sweep_rows * sweep_sets)), sblock(sweep_waves * 64);
    const bool sign = (gb[g] == 1 && prm.q1_mode == SLIM_Q1_SIGN);
#define SLIM_SWEEP4(B)                                                                           \
  do {                                                                                           \
    if (sign)                                                                                    \
      SLIM_LAUNCH(ctx, "gptq_sweep", (gptq_sweep4<B, true>), sgrid, sblock, sweep_smem, s);      \
    else                                                                                         \
      SLIM_LAUNCH(ctx, "gptq_sweep", (gptq_sweep4<B, false>), sgrid, sblock, sweep_smem, s);     \
  } while (0)
    if (SB == 32)
      SLIM_SWEEP4(32);
    else if (SB == 64)
      SLIM_SWEEP4(64);
    else
      SLIM_SWEEP4(128);
#undef SLIM_SWEEP4

    slim_gemm_desc d;
    d.C2 = nullptr;
    d.ldc2 = 0;
    d.M = n;
    d.flags = 0;
    d.alpha = -1.0;
    d.beta = 1.0;
    d.lda = WINC;
    d.ldb = ldu;
    d.ldc = m;
    if (b0 + SB < w1) {
      // the rest of the window
      d.A = E + (b0 - w0);
      d.B = U + (int64_t)b0 * ldu + (b0 + SB);
      d.C = Wc + (b0 + SB);
      d.N = w1 - (b0 + SB);
      d.K = SB;
      st = slim_dgemm(ctx, "gptq_window_dgemm", 0, d);
      if (st != SLIM_OK) return st;
    } else if (w1 < m) {
      // last block of the window: everything behind it
      d.A = E;
      d.B = U + (int64_t)w0 * ldu + w1;
      d.C = Wc + w1;
      d.N = m - w1;
      d.K = w1 - w0;
      st = slim_dgemm(ctx, "gptq_trailing_dgemm", 0, d);
      if (st != SLIM_OK) return st;
    }
  }
  if (sum_e2) return slim_sum_f64(ctx, "gptq_sum_e2", row_e2, n, sum_e2);
  return SLIM_OK;
}
