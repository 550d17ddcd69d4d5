// a3  Salience (Def. 1; Alg. 2 SBA line 6): column sums of w^2 divided by d_j^2, group means, and the
// optional element map.  A streaming kernel: W is read once (2 bytes per weight for fp16), sums are
// carried in fp64, partial sums per row slab are reduced in a fixed order so the result is
// deterministic.
#include "slim_device.h"
#include "slim_internal.h"

namespace {

using slimdev::load4;

// grid (ceil(m / 1024), nparts); thread -> 4 consecutive columns; part p owns rows [p*rpp, (p+1)*rpp).
// Rows are taken eight at a time with all eight loads issued before the first is used: the kernel is a stream
// over W, and a thread that waits for every row's load in turn leaves most of the memory system idle.
template <typename T, bool ELEM>
__global__ __launch_bounds__(256) void colsumsq_partial(const T* __restrict__ W, int n, int m, int64_t ldw,
                                                        int rows_per_part, const double* __restrict__ dden,
                                                        int64_t dstride, double* __restrict__ partial,
                                                        double* __restrict__ elem_sal) {
  const int c0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c0 >= m) return;
  const int r0 = blockIdx.y * rows_per_part;
  const int r1 = min(n, r0 + rows_per_part);
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  double inv[4] = {0.0, 0.0, 0.0, 0.0};
  if (ELEM) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double d = dden[(int64_t)(c0 + j) * dstride];
      inv[j] = d * d;
    }
  }
  constexpr int UR = 8;
  int r = r0;
  for (; r + UR <= r1; r += UR) {
    double w[UR][4];
#pragma unroll
    for (int u = 0; u < UR; ++u) load4<T>(W + (int64_t)(r + u) * ldw + c0, w[u]);
#pragma unroll
    for (int u = 0; u < UR; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const double sq = w[u][j] * w[u][j];
        acc[j] += sq;                                   // rows in order: the sum does not depend on the unrolling
        if (ELEM) elem_sal[(int64_t)(r + u) * m + c0 + j] = sq / inv[j];
      }
  }
  for (; r < r1; ++r) {
    double w[4];
    load4<T>(W + (int64_t)r * ldw + c0, w);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double sq = w[j] * w[j];
      acc[j] += sq;
      if (ELEM) elem_sal[(int64_t)r * m + c0 + j] = sq / inv[j];
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) partial[(int64_t)blockIdx.y * m + c0 + j] = acc[j];
}

// one workgroup per group g: col_sal for its beta columns, then the group mean.  The 1024 threads split the
// partial sums of a column among 1024 / beta slices (every slice-th part each), which are added in slice order.
__global__ __launch_bounds__(1024) void salience_finalize(const double* __restrict__ partial, int nparts, int n,
                                                          int m, int beta, const double* __restrict__ dden,
                                                          int64_t dstride, double* __restrict__ col_sal,
                                                          double* __restrict__ group_sal) {
  __shared__ double red[1024];
  const int g = blockIdx.x;
  const int cp = min(beta, 1024);               // columns per pass
  const int slices = 1024 / cp;
  const int jj = threadIdx.x % cp, sl = threadIdx.x / cp;
  double v = 0.0;                               // sum of the column saliences this thread finishes
  for (int j0 = 0; j0 < beta; j0 += cp) {
    const int j = j0 + jj;
    const int c = g * beta + j;
    double s = 0.0;
    if (sl < slices && j < beta)
      for (int p = sl; p < nparts; p += slices) s += partial[(int64_t)p * m + c];
    __syncthreads();
    red[threadIdx.x] = s;
    __syncthreads();
    if (sl == 0 && j < beta) {
      double t = 0.0;
      for (int q = 0; q < slices; ++q) t += red[q * cp + jj];
      const double d = dden[(int64_t)c * dstride];
      const double cs = t / (d * d);
      col_sal[c] = cs;
      v += cs;
    }
  }
  __syncthreads();
  red[threadIdx.x] = v;
  __syncthreads();
  for (int st = 512; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) group_sal[g] = red[0] / ((double)n * (double)beta);
}

}  // namespace

// row slabs of the partial column sums: about 2048 workgroups (eight per compute unit)
static void salience_parts(int n, int m, int& nparts, int& rpp) {
  const int gx = slim_cdiv(m, 1024);
  nparts = (2048 + gx - 1) / gx;
  if (nparts > n) nparts = n;
  rpp = slim_cdiv(n, nparts);
  nparts = slim_cdiv(n, rpp);
}

size_t slim_ws_need_salience(int n, int m) {
  int nparts = 0, rpp = 0;
  salience_parts(n, m, nparts, rpp);
  return slim_ws_round(sizeof(double) * (size_t)nparts * m);
}

extern "C" slim_status slim_salience(slim_ctx* ctx, const void* W, slim_dtype w_dtype, int n, int m, int64_t ldw,
                                     const double* U, int64_t ldu, const double* hinv_diag, int sal_mode,
                                     int beta, double* col_sal, double* group_sal, double* elem_sal) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, W && col_sal && group_sal, "slim_salience: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "slim_salience: need n, m > 0 and beta | m (n=%d m=%d beta=%d)", n, m, beta);
  SLIM_REQUIRE(ctx, m % 4 == 0 && ldw >= m && ldw % 4 == 0, "slim_salience: m and ldw must be multiples of 4");
  SLIM_REQUIRE(ctx, slim_aligned16(W), "slim_salience: W must be 16-byte aligned");
  const double* dden;
  int64_t dstride;
  if (sal_mode == SLIM_SAL_HINV_DIAG) {
    SLIM_REQUIRE(ctx, hinv_diag != nullptr, "slim_salience: hinv_diag is null");
    dden = hinv_diag;
    dstride = 1;
  } else if (sal_mode == SLIM_SAL_CHOL_DIAG) {
    SLIM_REQUIRE(ctx, U != nullptr && ldu >= m, "slim_salience: U is null or ldu < m");
    dden = U;
    dstride = ldu + 1;
  } else {
    return slim_fail(ctx, SLIM_ERR_INVALID_ARG, "slim_salience: unknown sal_mode %d", sal_mode);
  }
  if (w_dtype != SLIM_F16 && w_dtype != SLIM_BF16 && w_dtype != SLIM_F32)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_salience: W must be F16, BF16 or F32");

  const int gx = slim_cdiv(m, 1024);
  int nparts = 0, rpp = 0;
  salience_parts(n, m, nparts, rpp);
  slim_status st = slim_ws_reserve(ctx, slim_ws_need_salience(n, m));
  if (st != SLIM_OK) return st;
  double* partial = static_cast<double*>(slim_ws_alloc(ctx, sizeof(double) * (size_t)nparts * m));

  const dim3 grid(gx, nparts), block(256);
#define SLIM_COLSUMSQ(T, E)                                                                                      \
  SLIM_LAUNCH(ctx, "salience_colsumsq", (colsumsq_partial<T, E>), grid, block, 0, static_cast<const T*>(W), n, m, ldw, \
              rpp, dden, dstride, partial, elem_sal)
  if (w_dtype == SLIM_F16) {
    if (elem_sal) SLIM_COLSUMSQ(__half, true); else SLIM_COLSUMSQ(__half, false);
  } else if (w_dtype == SLIM_BF16) {
    if (elem_sal) SLIM_COLSUMSQ(__hip_bfloat16, true); else SLIM_COLSUMSQ(__hip_bfloat16, false);
  } else {
    if (elem_sal) SLIM_COLSUMSQ(float, true); else SLIM_COLSUMSQ(float, false);
  }
#undef SLIM_COLSUMSQ
  SLIM_LAUNCH(ctx, "salience_finalize", salience_finalize, dim3(m / beta), dim3(1024), 0, partial, nparts, n, m, beta,
              dden, dstride, col_sal, group_sal);
  return SLIM_OK;
}
