// fp64 GEMM on the CDNA matrix cores (v_mfma_f64_16x16x4_f64), used by every fp64 contraction of the
// pass: the trailing updates of the reverse Cholesky factorisation and of the triangular inverse
// (Alg. 1 line 2), the rank-beta trailing update of the GPTQ sweep (Alg. 1 line 12) and the layer
// outputs of the SBA objective (Eq. 4).
//
// Tiling: one 256-thread workgroup (4 wavefronts, 2 x 2) owns a BM x BN tile of C (128 x 128, or 64 x 64
// for problems too small to give every CU a big tile); every wavefront owns a quarter of it as MFMA tiles
// of 16 x 16.  K advances in slabs of 16 through two LDS buffers (k-major, so that the 16 lanes that feed
// one k-slice of an MFMA operand read 16 consecutive doubles); the next slab is fetched into registers
// while the current one is multiplied, one barrier per slab.
#include <algorithm>

#include "dgemm_device.h"
#include "slim_internal.h"

namespace {

using namespace slimgemm;

template <int BM, int BN>
struct Prefetch {
  double2 a[BM / 32];
  double2 b[BN / 32];
  unsigned va, vb;   // bit j set: element pair j is inside the matrix and the K range
};

// Loads are branch-free: an out-of-range element is read from a clamped (valid) address and replaced by
// zero only when it is written to LDS, so that the loads of the next slab stay in flight while the current
// slab is multiplied.
//
// Operand slab stored "rows x 16 k" in memory (A, or B when it is given as N x K): thread -> (row, part of
// the k range); R rows need R * 16 doubles = R / 32 double2 per thread.
template <int R>
__device__ __forceinline__ void load_rows_k(const double* base, int64_t ld, int nrows, int K, int row0, int k0,
                                            int kend, int tid, double2* out, unsigned& valid) {
  constexpr int PER = R / 32;                 // double2 per thread
  constexpr int TPR = 8 / PER;                // threads per row
  const int r = tid / TPR, kh = (tid % TPR) * (2 * PER);
  const int row = row0 + r;
  const bool rv = row < nrows;
  const double* src = base + (int64_t)min(row, nrows - 1) * ld;
  valid = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int k = k0 + kh + 2 * j;
    out[j] = *reinterpret_cast<const double2*>(src + min(k, K - 2));
    valid |= (rv && k < kend) ? (1u << j) : 0u;
  }
}

template <int R>
__device__ __forceinline__ void store_rows_k(double* S, int tid, const double2* in, unsigned valid) {
  constexpr int PER = R / 32;
  constexpr int TPR = 8 / PER;
  const int r = tid / TPR, kh = (tid % TPR) * (2 * PER);
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const bool v = (valid >> j) & 1u;
    S[(kh + 2 * j) * R + r] = v ? in[j].x : 0.0;
    S[(kh + 2 * j + 1) * R + r] = v ? in[j].y : 0.0;
  }
}

// B given as K x N: thread -> (k, consecutive n)
template <int BN>
__device__ __forceinline__ void load_k_cols(const double* base, int64_t ld, int N, int K, int col0, int k0, int kend,
                                            int tid, double2* out, unsigned& valid) {
  constexpr int PER = BN / 32;
  const int kk = tid >> 4, n0 = (tid & 15) * (2 * PER);
  const int k = k0 + kk;
  const bool kv = k < kend;
  const double* src = base + (int64_t)min(k, K - 1) * ld;
  valid = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const int col = col0 + n0 + 2 * j;
    out[j] = *reinterpret_cast<const double2*>(src + min(col, N - 2));
    valid |= (kv && col < N) ? (1u << j) : 0u;
  }
}

template <int BN>
__device__ __forceinline__ void store_k_cols(double* S, int tid, const double2* in, unsigned valid) {
  constexpr int PER = BN / 32;
  const int kk = tid >> 4, n0 = (tid & 15) * (2 * PER);
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const bool v = (valid >> j) & 1u;
    *reinterpret_cast<double2*>(&S[kk * BN + n0 + 2 * j]) = make_double2(v ? in[j].x : 0.0, v ? in[j].y : 0.0);
  }
}

// K loop with bounds handling (tiles on the matrix edges, K ranges that end inside a slab): loads from clamped
// addresses, zeros substituted on the way to LDS; fetch, multiply and stash are separate phases of an iteration.
template <int TRANS_B, int BM, int BN>
__device__ __forceinline__ void k_loop_edge(const slim_gemm_desc& d, int row0, int col0, int kbeg, int kend,
                                            double* smem, double4v (&acc)[BM / 32][BN / 32]) {
  constexpr int MI = BM / 32, NJ = BN / 32;
  constexpr int STAGE = BK * BM + BK * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l16 = lane & 15, lk = lane >> 4;
  Prefetch<BM, BN> pf;
  auto fetch = [&](int k0) {
    load_rows_k<BM>(d.A, d.lda, d.M, d.K, row0, k0, kend, tid, pf.a, pf.va);
    if (TRANS_B)
      load_rows_k<BN>(d.B, d.ldb, d.N, d.K, col0, k0, kend, tid, pf.b, pf.vb);
    else
      load_k_cols<BN>(d.B, d.ldb, d.N, d.K, col0, k0, kend, tid, pf.b, pf.vb);
  };
  auto stash = [&](double* st) {
    store_rows_k<BM>(st, tid, pf.a, pf.va);
    if (TRANS_B)
      store_rows_k<BN>(st + BK * BM, tid, pf.b, pf.vb);
    else
      store_k_cols<BN>(st + BK * BM, tid, pf.b, pf.vb);
  };

  int cur = 0;
  if (kbeg < kend) {
    fetch(kbeg);
    stash(smem);
  }
  __syncthreads();
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    // unconditional (the slab behind the last one is all zeros read from clamped addresses): one basic
    // block per iteration keeps the accumulators in place across the loop
    fetch(k0 + BK);
    __builtin_amdgcn_sched_barrier(0);   // keep the fetch ahead of, and its first use behind, the MFMA block
    const double* as = smem + cur * STAGE + wm * (BM / 2) + l16;
    const double* bs = smem + cur * STAGE + BK * BM + wn * (BN / 2) + l16;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 4) {
      double a[MI], b[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) a[i] = as[(kk + lk) * BM + i * 16];
#pragma unroll
      for (int j = 0; j < NJ; ++j) b[j] = bs[(kk + lk) * BN + j * 16];
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    stash(smem + (cur ^ 1) * STAGE);
    __syncthreads();
    cur ^= 1;
  }
}

template <int TRANS_B, int BM, int BN>
__device__ __forceinline__ void gemm_body(const slim_gemm_desc& d, int pid, double* smem) {
  constexpr int MI = BM / 32, NJ = BN / 32;   // MFMA tiles per wavefront along M and N
  const int tiles_n = (d.N + BN - 1) / BN;
  const int tiles_m = (d.M + BM - 1) / BM;
  if (pid >= tiles_m * tiles_n) return;
  // Tiles with the longest K range first.  With an upper triangular A those are the first rows, which come first
  // anyway.  With an upper triangular B they are the last columns: the tiles are then numbered column by column from
  // the last column, so that the tiles on the chip at one time have the same K range and end together (numbered row
  // by row, every row mixes K ranges from one slab to all of them, and a 4096^3 product of the triangular inverse
  // took 1.98 ms instead of 1.17).
  const bool colmajor = (d.flags & SLIM_GEMM_B_UPPER) != 0;
  const int bi = colmajor ? pid % tiles_m : pid / tiles_n;
  const int bj = colmajor ? tiles_n - 1 - pid / tiles_m : pid % tiles_n;
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

  double4v acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = double4v{0.0, 0.0, 0.0, 0.0};

  // Tiles inside both matrices whose K range is a whole number of slabs take the loop without bounds handling.
  const bool interior = row0 + BM <= d.M && col0 + BN <= d.N && (kend - kbeg) % BK == 0 && kend > kbeg;
  if (interior)
    k_loop_fast<TRANS_B, BM, BN>(d, row0, col0, kbeg, kend, smem, acc);
  else
    k_loop_edge<TRANS_B, BM, BN>(d, row0, col0, kbeg, kend, smem, acc);

  // Epilogue.  Accumulator register v of lane l holds C[4 * v + l / 16][l % 16] of its 16 x 16 tile.
  // The old values of C are fetched a row of MFMA tiles at a time (clamped addresses, no branches) before
  // any store, so that the read-modify-write costs one memory round trip per 16 rows instead of one per
  // element.
  const double alpha = d.alpha, beta = d.beta;
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    double cold[4][NJ];
    if (beta != 0.0) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = min(row0 + wm * (BM / 2) + i * 16 + 4 * v + lk, d.M - 1);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int col = min(col0 + wn * (BN / 2) + j * 16 + l16, d.N - 1);
          cold[v][j] = d.C[(int64_t)row * d.ldc + col];
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = row0 + wm * (BM / 2) + i * 16 + 4 * v + lk;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int col = col0 + wn * (BN / 2) + j * 16 + l16;
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

template <int TRANS_B, int BM, int BN>
__global__ __launch_bounds__(NTHREADS) void dgemm_kernel(slim_gemm_desc d) {
  extern __shared__ __align__(16) double smem[];
  gemm_body<TRANS_B, BM, BN>(d, blockIdx.x, smem);
}

template <int TRANS_B, int BM, int BN>
__global__ __launch_bounds__(NTHREADS) void dgemm_batched_kernel(const slim_gemm_desc* descs) {
  extern __shared__ __align__(16) double smem[];
  const slim_gemm_desc d = descs[blockIdx.y];
  gemm_body<TRANS_B, BM, BN>(d, blockIdx.x, smem);
}

// Persistent form for bulk work beside a latency-critical chain on another stream: fewer workgroups than CUs, each
// taking tiles in turn, with an LDS request that lets nothing else of any size share their CUs.  The CUs it leaves
// out stay free for the chain's kernels.  With SLIM_GEMM_UPPER_ONLY (M == N) only the tiles on or above the
// diagonal are enumerated.
template <int TRANS_B, int BM, int BN>
__global__ __launch_bounds__(NTHREADS) void dgemm_reserved_kernel(slim_gemm_desc d) {
  extern __shared__ __align__(16) double smem[];
  const int tiles_n = (d.N + BN - 1) / BN, tiles_m = (d.M + BM - 1) / BM;
  if (d.flags & SLIM_GEMM_UPPER_ONLY) {
    const int nt = tiles_n;                       // square: tiles_m == tiles_n
    const int total = nt * (nt + 1) / 2;
    for (int u = blockIdx.x; u < total; u += gridDim.x) {
      // row bi holds the nt - bi tiles bj >= bi; rows before it hold bi * nt - bi (bi - 1) / 2
      int bi = (int)((2.0f * nt + 1.0f - sqrtf((2.0f * nt + 1.0f) * (2.0f * nt + 1.0f) - 8.0f * u)) * 0.5f);
      bi = max(0, min(bi, nt - 1));
      while (bi > 0 && bi * nt - bi * (bi - 1) / 2 > u) --bi;
      while (bi + 1 < nt && (bi + 1) * nt - (bi + 1) * bi / 2 <= u) ++bi;
      const int bj = bi + (u - (bi * nt - bi * (bi - 1) / 2));
      gemm_body<TRANS_B, BM, BN>(d, bi * tiles_n + bj, smem);
    }
  } else {
    for (int pid = blockIdx.x; pid < tiles_m * tiles_n; pid += gridDim.x) gemm_body<TRANS_B, BM, BN>(d, pid, smem);
  }
}

// The same for products without edges (M a multiple of 256, N of 128, K of 16, no flags): 512 threads per
// workgroup on a 256 x 128 tile, so that the one workgroup a CU holds still gives every SIMD two wavefronts.
// Up to two products share a launch: their tiles are numbered through, which evens out the last round.
struct WidePair {
  slim_gemm_desc d[2];
  int count;
};
template <int TRANS_B>
__global__ __launch_bounds__(512) void dgemm_reserved_wide_kernel(WidePair w) {
  constexpr int BM = 256, BN = 128, NT = 512, MI = 4, NJ = 4;
  extern __shared__ __align__(16) double smem[];
  const int tiles0 = (w.d[0].M / BM) * (w.d[0].N / BN);
  const int tiles = tiles0 + (w.count > 1 ? (w.d[1].M / BM) * (w.d[1].N / BN) : 0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1, l16 = lane & 15, lk = lane >> 4;
  for (int unit = blockIdx.x; unit < tiles; unit += gridDim.x) {
    const slim_gemm_desc& d = unit < tiles0 ? w.d[0] : w.d[1];
    const int pid = unit < tiles0 ? unit : unit - tiles0;
    const int tiles_n = d.N / BN;
    const int row0 = (pid / tiles_n) * BM, col0 = (pid % tiles_n) * BN;
    double4v acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = double4v{0.0, 0.0, 0.0, 0.0};
    k_loop_fast<TRANS_B, BM, BN, NT>(d, row0, col0, 0, d.K, smem, acc);
    // accumulator register v of lane l holds C[4 * v + l / 16][l % 16] of its 16 x 16 tile
    const double alpha = d.alpha, beta = d.beta;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        double* crow = d.C + (int64_t)(row0 + wm * 64 + i * 16 + 4 * v + lk) * d.ldc + col0 + wn * 64 + l16;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          double r = alpha * acc[i][j][v];
          if (beta != 0.0) r += beta * crow[j * 16];
          crow[j * 16] = r;
        }
      }
  }
}

constexpr size_t smem_bytes(int bm, int bn) { return size_t(2) * (BK * bm + BK * bn) * sizeof(double); }

// 64 x 64 tiles when 128 x 128 tiles would leave most of the 256 CUs without work
bool use_small_tiles(int M, int N, int count) {
  return (int64_t)slim_cdiv(M, 128) * slim_cdiv(N, 128) * count < 192;
}

slim_status check_desc(slim_ctx* ctx, const slim_gemm_desc& d) {
  SLIM_REQUIRE(ctx, d.M >= 0 && d.N >= 0 && d.K >= 0, "dgemm: negative size");
  if (d.M == 0 || d.N == 0) return SLIM_OK;
  SLIM_REQUIRE(ctx, d.K >= 2, "dgemm: K must be at least 2");
  SLIM_REQUIRE(ctx, (d.K % 2) == 0 && (d.N % 2) == 0, "dgemm: K and N must be even (K=%d N=%d)", d.K, d.N);
  SLIM_REQUIRE(ctx, (d.lda % 2) == 0 && (d.ldb % 2) == 0 && (d.ldc % 2) == 0, "dgemm: odd leading dimension");
  SLIM_REQUIRE(ctx, slim_aligned16(d.A) && slim_aligned16(d.B) && slim_aligned16(d.C), "dgemm: misaligned pointer");
  return SLIM_OK;
}

// The persistent form asks for all of a CU's LDS (160 KiB), so nothing else shares its CUs, and leaves RESERVED_CUS
// of them alone: room for the chain's own kernels and the small products it waits for.
constexpr size_t ONE_PER_CU_BYTES = 160 * 1024;
constexpr int RESERVED_CUS = 32;

template <typename K>
slim_status allow_lds(slim_ctx* ctx, K kernel, bool& done) {
  if (!done) {
    SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)ONE_PER_CU_BYTES));
    done = true;
  }
  return SLIM_OK;
}

}  // namespace

slim_status slim_dgemm(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc& d) {
  slim_status st = check_desc(ctx, d);
  if (st != SLIM_OK) return st;
  if (d.M == 0 || d.N == 0) return SLIM_OK;
  if (d.flags & SLIM_GEMM_CHAIN) {
    const int tiles = slim_cdiv(d.M, 64) * slim_cdiv(d.N, 32);
    if (trans_b)
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<1, 64, 32>"), (dgemm_kernel<1, 64, 32>), dim3(tiles),
                  dim3(NTHREADS), smem_bytes(64, 32), d);
    else
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<0, 64, 32>"), (dgemm_kernel<0, 64, 32>), dim3(tiles),
                  dim3(NTHREADS), smem_bytes(64, 32), d);
    return SLIM_OK;
  }
  if (use_small_tiles(d.M, d.N, 1)) {
    const int tiles = slim_cdiv(d.M, 64) * slim_cdiv(d.N, 64);
    if (trans_b)
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<1, 64, 64>"), (dgemm_kernel<1, 64, 64>), dim3(tiles),
                  dim3(NTHREADS), smem_bytes(64, 64), d);
    else
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<0, 64, 64>"), (dgemm_kernel<0, 64, 64>), dim3(tiles),
                  dim3(NTHREADS), smem_bytes(64, 64), d);
    return SLIM_OK;
  }
  const int tiles = slim_cdiv(d.M, 128) * slim_cdiv(d.N, 128);
  const size_t lds = smem_bytes(128, 128);
  if (d.flags & SLIM_GEMM_ONE_PER_CU) {
    static bool done0 = false, done1 = false;
    st = trans_b ? allow_lds(ctx, dgemm_reserved_kernel<1, 128, 128>, done1)
                 : allow_lds(ctx, dgemm_reserved_kernel<0, 128, 128>, done0);
    if (st != SLIM_OK) return st;
    int work = tiles;
    if (d.flags & SLIM_GEMM_UPPER_ONLY) {
      SLIM_REQUIRE(ctx, d.M == d.N, "dgemm: SLIM_GEMM_UPPER_ONLY needs a square result");
      const int nt = slim_cdiv(d.N, 128);
      work = nt * (nt + 1) / 2;
    }
    const int wgs = std::max(1, std::min(work, ctx->num_cus - RESERVED_CUS));
    if (trans_b)
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_reserved_kernel<1, 128, 128>"), (dgemm_reserved_kernel<1, 128, 128>),
                  dim3(wgs), dim3(NTHREADS), ONE_PER_CU_BYTES, d);
    else
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_reserved_kernel<0, 128, 128>"), (dgemm_reserved_kernel<0, 128, 128>),
                  dim3(wgs), dim3(NTHREADS), ONE_PER_CU_BYTES, d);
    return SLIM_OK;
  }
  // 128 x 128 tiles, two to a CU, or 128 x 64 tiles, three to a CU and a little less efficient each: whichever
  // fills the rounds of workgroups better.  Cost of a form = rounds x (tile area x tiles per CU / efficiency).
  const int cus = std::max(1, ctx->num_cus);
  const int tiles_n64 = slim_cdiv(d.M, 128) * slim_cdiv(d.N, 64);
  const double cost128 = slim_cdiv(tiles, 2 * cus) * (128.0 * 128.0 * 2 / 0.91);
  const double cost64 = slim_cdiv(tiles_n64, 3 * cus) * (128.0 * 64.0 * 3 / 0.85);
  if (!(d.flags & SLIM_GEMM_UPPER_ONLY) && cost64 < cost128) {
    if (trans_b)
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<1, 128, 64>"), (dgemm_kernel<1, 128, 64>), dim3(tiles_n64),
                  dim3(NTHREADS), smem_bytes(128, 64), d);
    else
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<0, 128, 64>"), (dgemm_kernel<0, 128, 64>), dim3(tiles_n64),
                  dim3(NTHREADS), smem_bytes(128, 64), d);
    return SLIM_OK;
  }
  if (trans_b)
    SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<1, 128, 128>"), (dgemm_kernel<1, 128, 128>), dim3(tiles),
                dim3(NTHREADS), lds, d);
  else
    SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_kernel<0, 128, 128>"), (dgemm_kernel<0, 128, 128>), dim3(tiles),
                dim3(NTHREADS), lds, d);
  return SLIM_OK;
}

slim_status slim_dgemm_reserved(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc* descs, int count,
                                int cus) {
  if (count < 1 || count > 2) return slim_fail(ctx, SLIM_ERR_INVALID_ARG, "dgemm: one or two products per reserved launch");
  if (cus < 1 || cus > ctx->num_cus) return slim_fail(ctx, SLIM_ERR_INVALID_ARG, "dgemm: reserved launch on %d CUs", cus);
  bool wide = true;
  int tiles = 0;
  for (int i = 0; i < count; ++i) {
    const slim_gemm_desc& d = descs[i];
    slim_status st = check_desc(ctx, d);
    if (st != SLIM_OK) return st;
    wide = wide && d.flags == 0 && d.M > 0 && d.N > 0 && d.M % 256 == 0 && d.N % 128 == 0 && d.K % 16 == 0 && d.K > 0 && !d.C2;
    if (wide) tiles += (d.M / 256) * (d.N / 128);
  }
  if (!wide) {
    for (int i = 0; i < count; ++i) {
      slim_gemm_desc d = descs[i];
      d.flags |= SLIM_GEMM_ONE_PER_CU;
      slim_status st = slim_dgemm(ctx, name, trans_b, d);
      if (st != SLIM_OK) return st;
    }
    return SLIM_OK;
  }
  static bool wide0 = false, wide1 = false;
  slim_status st = trans_b ? allow_lds(ctx, dgemm_reserved_wide_kernel<1>, wide1) : allow_lds(ctx, dgemm_reserved_wide_kernel<0>, wide0);
  if (st != SLIM_OK) return st;
  // as many rounds as the CUs that may be used need, and then no more workgroups than fill those rounds
  const int usable = cus;
  const int rounds = slim_cdiv(tiles, usable);
  const int wgs = slim_cdiv(tiles, rounds);
  WidePair w;
  w.d[0] = descs[0];
  w.d[1] = descs[count - 1];
  w.count = count;
  if (trans_b)
    SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_reserved_wide_kernel<1>"), (dgemm_reserved_wide_kernel<1>), dim3(wgs),
                dim3(512), ONE_PER_CU_BYTES, w);
  else
    SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_reserved_wide_kernel<0>"), (dgemm_reserved_wide_kernel<0>), dim3(wgs),
                dim3(512), ONE_PER_CU_BYTES, w);
  return SLIM_OK;
}

slim_status slim_dgemm_batched(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc* descs_dev,
                               int count, int max_M, int max_N) {
  if (count == 0 || max_M == 0 || max_N == 0) return SLIM_OK;
  // The products of a batch have triangular operands, so the K ranges of their tiles differ by large factors: up to
  // two rounds of 128 x 128 tiles would last as long as the longest tile, while many 64 x 64 tiles per CU even out.
  const bool uneven = (int64_t)slim_cdiv(max_M, 128) * slim_cdiv(max_N, 128) * count <= 2 * (int64_t)ctx->num_cus;
  if (uneven || use_small_tiles(max_M, max_N, count)) {
    const int tiles = slim_cdiv(max_M, 64) * slim_cdiv(max_N, 64);
    if (trans_b)
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_batched_kernel<1, 64, 64>"), (dgemm_batched_kernel<1, 64, 64>),
                  dim3(tiles, count), dim3(NTHREADS), smem_bytes(64, 64), descs_dev);
    else
      SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_batched_kernel<0, 64, 64>"), (dgemm_batched_kernel<0, 64, 64>),
                  dim3(tiles, count), dim3(NTHREADS), smem_bytes(64, 64), descs_dev);
    return SLIM_OK;
  }
  const int tiles = slim_cdiv(max_M, 128) * slim_cdiv(max_N, 128);
  if (trans_b)
    SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_batched_kernel<1, 128, 128>"), (dgemm_batched_kernel<1, 128, 128>),
                dim3(tiles, count), dim3(NTHREADS), smem_bytes(128, 128), descs_dev);
  else
    SLIM_LAUNCH(ctx, slim_prof_name(name, "dgemm_batched_kernel<0, 128, 128>"), (dgemm_batched_kernel<0, 128, 128>),
                dim3(tiles, count), dim3(NTHREADS), smem_bytes(128, 128), descs_dev);
  return SLIM_OK;
}
