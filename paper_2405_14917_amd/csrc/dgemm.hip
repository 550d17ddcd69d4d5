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
  unsigned va, vb;   // bit j set: element pair j is inside the matrix and the K range
};

// Loads are branch-free: an out-of-range element is read from a clamped (valid) address and replaced by
// zero only when it is written to LDS, so that the loads of the next slab stay in flight while the current
// slab is multiplied.
template <int TRANS_B>
__device__ __forceinline__ void load_global(const slim_gemm_desc& d, int row0, int col0, int k0, int kend,
                                            int tid, Prefetch& p) {
  p.va = 0;
  p.vb = 0;
  // A slab: 128 rows x 16 k.  Thread -> (row, half of the k range), 4 x 16 bytes contiguous in k.
  {
    const int r = tid >> 1, kh = (tid & 1) * 8;
    const int row = row0 + r;
    const bool rv = row < d.M;
    const double* src = d.A + (int64_t)min(row, d.M - 1) * d.lda;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + kh + 2 * j;
      p.a[j] = *reinterpret_cast<const double2*>(src + min(k, d.K - 2));
      p.va |= (rv && k < kend) ? (1u << j) : 0u;
    }
  }
  if (TRANS_B) {
    // B stored N x K: same pattern as A with n in the role of the row
    const int r = tid >> 1, kh = (tid & 1) * 8;
    const int col = col0 + r;
    const bool cv = col < d.N;
    const double* src = d.B + (int64_t)min(col, d.N - 1) * d.ldb;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + kh + 2 * j;
      p.b[j] = *reinterpret_cast<const double2*>(src + min(k, d.K - 2));
      p.vb |= (cv && k < kend) ? (1u << j) : 0u;
    }
  } else {
    // B stored K x N: thread -> (k, 8 consecutive n)
    const int kk = tid >> 4, n0 = (tid & 15) * 8;
    const int k = k0 + kk;
    const bool kv = k < kend;
    const double* src = d.B + (int64_t)min(k, d.K - 1) * d.ldb;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = col0 + n0 + 2 * j;
      p.b[j] = *reinterpret_cast<const double2*>(src + min(col, d.N - 2));
      p.vb |= (kv && col < d.N) ? (1u << j) : 0u;
    }
  }
}

template <int TRANS_B>
__device__ __forceinline__ void store_lds(double* As, double* Bs, int tid, const Prefetch& p) {
  {
    const int r = tid >> 1, kh = (tid & 1) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool v = (p.va >> j) & 1u;
      As[(kh + 2 * j) * BM + r] = v ? p.a[j].x : 0.0;
      As[(kh + 2 * j + 1) * BM + r] = v ? p.a[j].y : 0.0;
    }
  }
  if (TRANS_B) {
    const int r = tid >> 1, kh = (tid & 1) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool v = (p.vb >> j) & 1u;
      Bs[(kh + 2 * j) * BN + r] = v ? p.b[j].x : 0.0;
      Bs[(kh + 2 * j + 1) * BN + r] = v ? p.b[j].y : 0.0;
    }
  } else {
    const int kk = tid >> 4, n0 = (tid & 15) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool v = (p.vb >> j) & 1u;
      *reinterpret_cast<double2*>(&Bs[kk * BN + n0 + 2 * j]) = make_double2(v ? p.b[j].x : 0.0, v ? p.b[j].y : 0.0);
    }
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

  // LDS stage s: A slab at smem + s * STAGE, B slab BK * BM behind it (plain offsets from one base keep the
  // accesses in the LDS address space)
  constexpr int STAGE = BK * BM + BK * BN;

  double4v acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = double4v{0.0, 0.0, 0.0, 0.0};

  Prefetch pf;
  int cur = 0;
  if (kbeg < kend) {
    load_global<TRANS_B>(d, row0, col0, kbeg, kend, tid, pf);
    store_lds<TRANS_B>(smem, smem + BK * BM, tid, pf);
  }
  __syncthreads();
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    // unconditional (the slab behind the last one is all zeros read from clamped addresses): one basic
    // block per iteration keeps the accumulators in place across the loop
    load_global<TRANS_B>(d, row0, col0, k0 + BK, kend, tid, pf);
    __builtin_amdgcn_sched_barrier(0);   // keep the fetch ahead of, and its first use behind, the MFMA block
    const double* as = smem + cur * STAGE + wm * 64 + l16;
    const double* bs = smem + cur * STAGE + BK * BM + wn * 64 + l16;
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
    __builtin_amdgcn_sched_barrier(0);
    store_lds<TRANS_B>(smem + (cur ^ 1) * STAGE, smem + (cur ^ 1) * STAGE + BK * BM, tid, pf);
    __syncthreads();
    cur ^= 1;
  }

  // Epilogue.  Accumulator register v of lane l holds C[4 * v + l / 16][l % 16] of its 16 x 16 tile.
  // The old values of C are fetched 16 at a time (clamped addresses, no branches) before any store, so
  // that the read-modify-write costs one memory round trip per 16 rows instead of one per element.
  const double alpha = d.alpha, beta = d.beta;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    double cold[4][4];
    if (beta != 0.0) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = min(row0 + wm * 64 + i * 16 + 4 * v + lk, d.M - 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int col = min(col0 + wn * 64 + j * 16 + l16, d.N - 1);
          cold[v][j] = d.C[(int64_t)row * d.ldc + col];
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = row0 + wm * 64 + i * 16 + 4 * v + lk;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = col0 + wn * 64 + j * 16 + l16;
        double r = alpha * acc[i][j][v];
        if (beta != 0.0) r += beta * cold[v][j];
        if (row < d.M && col < d.N) {
          d.C[(int64_t)row * d.ldc + col] = r;
          if (d.C2) d.C2[(int64_t)row * d.ldc2 + col] = r;
        }
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
  if (d.M == 0 || d.N == 0) return SLIM_OK;
  SLIM_REQUIRE(ctx, d.K >= 2, "dgemm: K must be at least 2");
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
