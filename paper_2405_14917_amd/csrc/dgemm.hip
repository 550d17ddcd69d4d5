// fp64 GEMM on the CDNA matrix cores (v_mfma_f64_16x16x4_f64), used by every fp64 contraction of the
// pass: the trailing updates of the reverse Cholesky factorisation and of the triangular inverse
// (Alg. 1 line 2), the rank-beta trailing update of the GPTQ sweep (Alg. 1 line 12) and the layer
// outputs of the SBA objective (Eq. 4).
//
// Tiling: one 256-thread workgroup (4 wavefronts, 2 x 2) owns a 128 x 128 tile of C; every wavefront
// owns 64 x 64 of it as 4 x 4 MFMA tiles of 16 x 16 (128 accumulator registers per lane).  K advances
// in slabs of 16 through two LDS buffers (k-major, so that the 16 lanes that feed one k-slice of an
// MFMA operand read 16 consecutive doubles); the next slab is fetched into registers while the
// current one is multiplied, one barrier per slab.
#include "slim_internal.h"

namespace {

typedef double double4v __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16, NTHREADS = 256;

struct Prefetch {
  double2 a[4];
  double2 b[4];
};

template <int TRANS_B>
__device__ __forceinline__ void load_global(const slim_gemm_desc& d, int row0, int col0, int k0, int kend,
                                            int tid, Prefetch& p) {
  // A slab: 128 rows x 16 k.  Thread -> (row, half of the k range), 4 x 16 bytes contiguous in k.
  {
    const int r = tid >> 1, kh = (tid & 1) * 8;
    const int row = row0 + r;
    const double* src = d.A + (int64_t)row * d.lda + k0 + kh;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + kh + 2 * j;
      p.a[j] = (row < d.M && k < kend) ? *reinterpret_cast<const double2*>(src + 2 * j) : make_double2(0.0, 0.0);
    }
  }
  if (TRANS_B) {
    // B stored N x K: same pattern as A with n in the role of the row
    const int r = tid >> 1, kh = (tid & 1) * 8;
    const int col = col0 + r;
    const double* src = d.B + (int64_t)col * d.ldb + k0 + kh;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + kh + 2 * j;
      p.b[j] = (col < d.N && k < kend) ? *reinterpret_cast<const double2*>(src + 2 * j) : make_double2(0.0, 0.0);
    }
  } else {
    // B stored K x N: thread -> (k, 8 consecutive n)
    const int kk = tid >> 4, n0 = (tid & 15) * 8;
    const int k = k0 + kk;
    const double* src = d.B + (int64_t)k * d.ldb + col0 + n0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = col0 + n0 + 2 * j;
      p.b[j] = (k < kend && col < d.N) ? *reinterpret_cast<const double2*>(src + 2 * j) : make_double2(0.0, 0.0);
    }
  }
}

template <int TRANS_B>
__device__ __forceinline__ void store_lds(double* As, double* Bs, int tid, const Prefetch& p) {
  {
    const int r = tid >> 1, kh = (tid & 1) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      As[(kh + 2 * j) * BM + r] = p.a[j].x;
      As[(kh + 2 * j + 1) * BM + r] = p.a[j].y;
    }
  }
  if (TRANS_B) {
    const int r = tid >> 1, kh = (tid & 1) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      Bs[(kh + 2 * j) * BN + r] = p.b[j].x;
      Bs[(kh + 2 * j + 1) * BN + r] = p.b[j].y;
    }
  } else {
    const int kk = tid >> 4, n0 = (tid & 15) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<double2*>(&Bs[kk * BN + n0 + 2 * j]) = p.b[j];
  }
}

template <int TRANS_B>
__device__ __forceinline__ void gemm_body(const slim_gemm_desc& d, int pid, double* smem) {
  const int tiles_n = (d.N + BN - 1) / BN;
  const int tiles_m = (d.M + BM - 1) / BM;
  if (pid >= tiles_m * tiles_n) return;
  const int bi = pid / tiles_n, bj = pid % tiles_n;
  const int row0 = bi * BM, col0 = bj * BN;
  if ((d.flags & SLIM_GEMM_UPPER_ONLY) && row0 >= col0 + BN) return;

  int kbeg = 0, kend = d.K;
  if (d.flags & SLIM_GEMM_A_UPPER) kbeg = (row0 / BK) * BK;              // A[i][k] = 0 for k < i
  if (d.flags & SLIM_GEMM_B_UPPER) kend = min(d.K, col0 + BN);           // B[k][n] = 0 for k > n

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l16 = lane & 15, lk = lane >> 4;

  double* As[2] = {smem, smem + BK * BM + BK * BN};
  double* Bs[2] = {smem + BK * BM, smem + 2 * BK * BM + BK * BN};

  double4v acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = double4v{0.0, 0.0, 0.0, 0.0};

  Prefetch pf;
  int cur = 0;
  if (kbeg < kend) {
    load_global<TRANS_B>(d, row0, col0, kbeg, kend, tid, pf);
    store_lds<TRANS_B>(As[0], Bs[0], tid, pf);
  }
  __syncthreads();
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    const bool more = k0 + BK < kend;
    if (more) load_global<TRANS_B>(d, row0, col0, k0 + BK, kend, tid, pf);
    const double* as = As[cur] + wm * 64 + l16;
    const double* bs = Bs[cur] + wn * 64 + l16;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 4) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = as[(kk + lk) * BM + i * 16];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = bs[(kk + lk) * BN + j * 16];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (more) store_lds<TRANS_B>(As[cur ^ 1], Bs[cur ^ 1], tid, pf);
    __syncthreads();
    cur ^= 1;
  }

  // Epilogue.  Accumulator register v of lane l holds C[4 * v + l / 16][l % 16] of its 16 x 16 tile.
  const double alpha = d.alpha, beta = d.beta;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = row0 + wm * 64 + i * 16 + 4 * v + lk;
      if (row >= d.M) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = col0 + wn * 64 + j * 16 + l16;
        if (col >= d.N) continue;
        double r = alpha * acc[i][j][v];
        double* c = d.C + (int64_t)row * d.ldc + col;
        if (beta != 0.0) r += beta * (*c);
        *c = r;
        if (d.C2) d.C2[(int64_t)row * d.ldc2 + col] = r;
      }
    }
  }
}

template <int TRANS_B>
__global__ __launch_bounds__(NTHREADS) void dgemm_kernel(slim_gemm_desc d) {
  extern __shared__ __align__(16) double smem[];
  gemm_body<TRANS_B>(d, blockIdx.x, smem);
}

template <int TRANS_B>
__global__ __launch_bounds__(NTHREADS) void dgemm_batched_kernel(const slim_gemm_desc* descs) {
  extern __shared__ __align__(16) double smem[];
  const slim_gemm_desc d = descs[blockIdx.y];
  gemm_body<TRANS_B>(d, blockIdx.x, smem);
}

constexpr size_t kSmemBytes = size_t(2) * (BK * BM + BK * BN) * sizeof(double);

slim_status check_desc(slim_ctx* ctx, const slim_gemm_desc& d) {
  SLIM_REQUIRE(ctx, d.M >= 0 && d.N >= 0 && d.K >= 0, "dgemm: negative size");
  SLIM_REQUIRE(ctx, (d.K % 2) == 0 && (d.N % 2) == 0, "dgemm: K and N must be even (K=%d N=%d)", d.K, d.N);
  SLIM_REQUIRE(ctx, (d.lda % 2) == 0 && (d.ldb % 2) == 0 && (d.ldc % 2) == 0, "dgemm: odd leading dimension");
  SLIM_REQUIRE(ctx, slim_aligned16(d.A) && slim_aligned16(d.B) && slim_aligned16(d.C), "dgemm: misaligned pointer");
  return SLIM_OK;
}

}  // namespace

slim_status slim_dgemm(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc& d) {
  slim_status st = check_desc(ctx, d);
  if (st != SLIM_OK) return st;
  if (d.M == 0 || d.N == 0) return SLIM_OK;
  const int tiles = slim_cdiv(d.M, BM) * slim_cdiv(d.N, BN);
  if (trans_b)
    SLIM_LAUNCH(ctx, name, dgemm_kernel<1>, dim3(tiles), dim3(NTHREADS), kSmemBytes, d);
  else
    SLIM_LAUNCH(ctx, name, dgemm_kernel<0>, dim3(tiles), dim3(NTHREADS), kSmemBytes, d);
  return SLIM_OK;
}

slim_status slim_dgemm_batched(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc* descs_dev,
                               int count, int max_M, int max_N) {
  if (count == 0 || max_M == 0 || max_N == 0) return SLIM_OK;
  const int tiles = slim_cdiv(max_M, BM) * slim_cdiv(max_N, BN);
  if (trans_b)
    SLIM_LAUNCH(ctx, name, dgemm_batched_kernel<1>, dim3(tiles, count), dim3(NTHREADS), kSmemBytes, descs_dev);
  else
    SLIM_LAUNCH(ctx, name, dgemm_batched_kernel<0>, dim3(tiles, count), dim3(NTHREADS), kSmemBytes, descs_dev);
  return SLIM_OK;
}
