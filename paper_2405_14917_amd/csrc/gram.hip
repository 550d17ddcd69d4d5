// a1  Proxy Hessian (Eq. 3; Alg. 1 line 1):  G += X_c X_c^T  on the fp16 / bf16 matrix cores
// (v_mfma_f32_32x32x16), fp32 accumulation.
//
// X is m x t with tokens contiguous, so both operands of X X^T are K-contiguous and the kernel is an
// "NT" product of X with itself.  Only tile pairs (bi <= bj) of the symmetric result are computed.
//
//  * Workgroup tile 256 x 256, 256 threads = 4 wavefronts in 2 x 2, each owning 128 x 128 as 4 x 4 MFMA
//    tiles of 32 x 32 (256 fp32 accumulators per lane).  Per K step of 16 a wavefront reads 8 operand
//    fragments from LDS for 16 MFMAs, which keeps LDS at about half of its bandwidth.
//  * K advances in slabs of 64 tokens (128 bytes per row = one cache line) through two LDS stages;
//    the next slab is fetched into registers while the current one is multiplied; rows are padded to
//    72 halves so that the 16-byte operand reads of consecutive rows fall into different banks.
//  * Split-K: workgroup id = tile * S + s.  Workgroups are dealt round-robin to the 8 XCDs, so with S a
//    multiple of 8 every XCD works on one token range and the slab of X that all of its tiles share
//    stays in that XCD's L2.
//  * Each split writes its partial tile to a scratch buffer; a second kernel adds the partials to G in
//    a fixed order (deterministic, no floating-point atomics) and mirrors the upper triangle.
#include "slim_internal.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int TM = 256;            // tile edge
constexpr int BK = 64;             // tokens per slab
constexpr int LDS_STRIDE = BK + 8; // halves per LDS row
constexpr int NTHREADS = 256;
constexpr int CHUNKS = TM * (BK / 8) / NTHREADS;  // 16-byte chunks per thread and operand = 8
constexpr size_t kSmemBytes = size_t(2) * 2 * TM * LDS_STRIDE * sizeof(uint16_t);

struct GramArgs {
  const uint16_t* X;   // 16-bit elements, m x t, ld = ldx
  int64_t ldx;
  int m;
  int64_t t;           // tokens in this chunk
  int64_t kchunk;      // tokens per split (multiple of BK)
  int S;               // number of splits
  float* P;            // partials: [S][m][m]
};

__device__ __forceinline__ void decode_tile(int t, int& bi, int& bj) {
  int j = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
  while ((j + 1) * (j + 2) / 2 <= t) ++j;
  while (j * (j + 1) / 2 > t) --j;
  bj = j;
  bi = t - j * (j + 1) / 2;
}

// 8 consecutive 16-bit elements of row `row` starting at token k; zero outside the matrix / the chunk.
__device__ __forceinline__ uint4 load_chunk(const GramArgs& a, int row, int64_t k, int64_t kend) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row >= a.m || k >= kend) return v;
  const uint16_t* p = a.X + (int64_t)row * a.ldx + k;
  if (k + 8 <= kend) return *reinterpret_cast<const uint4*>(p);
  uint16_t tmp[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int e = 0; e < 8; ++e)
    if (k + e < kend) tmp[e] = p[e];
  v.x = tmp[0] | ((uint32_t)tmp[1] << 16);
  v.y = tmp[2] | ((uint32_t)tmp[3] << 16);
  v.z = tmp[4] | ((uint32_t)tmp[5] << 16);
  v.w = tmp[6] | ((uint32_t)tmp[7] << 16);
  return v;
}

template <bool BF16>
__device__ __forceinline__ float16v mfma(const uint4& a, const uint4& b, float16v c) {
  if constexpr (BF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(&a),
                                                   *reinterpret_cast<const bf16x8*>(&b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const half8*>(&a),
                                                  *reinterpret_cast<const half8*>(&b), c, 0, 0, 0);
  }
}

template <bool BF16>
__global__ __launch_bounds__(NTHREADS) void gram_kernel(GramArgs a) {
  extern __shared__ __align__(16) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int split = blockIdx.x % a.S;
  int bi, bj;
  decode_tile(blockIdx.x / a.S, bi, bj);
  const int rowA0 = bi * TM, rowB0 = bj * TM;
  const int64_t kbeg = (int64_t)split * a.kchunk;
  const int64_t kend = min(a.t, kbeg + a.kchunk);

  // stage s: A slab at smem + s * STAGE, B slab TM * LDS_STRIDE behind it
  constexpr int STAGE = 2 * TM * LDS_STRIDE;

  float16v acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 pa[CHUNKS], pb[CHUNKS];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int id = c * NTHREADS + tid;
      const int r = id >> 3, ch = id & 7;
      pa[c] = load_chunk(a, rowA0 + r, k0 + ch * 8, kend);
      pb[c] = load_chunk(a, rowB0 + r, k0 + ch * 8, kend);
    }
  };
  auto stash = [&](uint16_t* as, uint16_t* bs) {
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int id = c * NTHREADS + tid;
      const int r = id >> 3, ch = id & 7;
      *reinterpret_cast<uint4*>(as + r * LDS_STRIDE + ch * 8) = pa[c];
      *reinterpret_cast<uint4*>(bs + r * LDS_STRIDE + ch * 8) = pb[c];
    }
  };

  int cur = 0;
  if (kbeg < kend) {
    fetch(kbeg);
    stash(smem, smem + TM * LDS_STRIDE);
  }
  __syncthreads();
  const int l32 = lane & 31, lh = lane >> 5;
  for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
    const bool more = k0 + BK < kend;
    if (more) fetch(k0 + BK);
    const uint16_t* as = smem + cur * STAGE + (wm * 128 + l32) * LDS_STRIDE + lh * 8;
    const uint16_t* bs = smem + cur * STAGE + TM * LDS_STRIDE + (wn * 128 + l32) * LDS_STRIDE + lh * 8;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      uint4 fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const uint4*>(as + i * 32 * LDS_STRIDE + kk);
#pragma unroll
      for (int j = 0; j < 4; ++j) fb[j] = *reinterpret_cast<const uint4*>(bs + j * 32 * LDS_STRIDE + kk);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mfma<BF16>(fa[i], fb[j], acc[i][j]);
    }
    if (more) stash(smem + (cur ^ 1) * STAGE, smem + (cur ^ 1) * STAGE + TM * LDS_STRIDE);
    __syncthreads();
    cur ^= 1;
  }

  // Accumulator register v of lane l holds C[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32] of its 32 x 32 tile.
  float* P = a.P + (int64_t)split * a.m * a.m;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = rowA0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
      if (row >= a.m) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = rowB0 + wn * 128 + j * 32 + l32;
        if (col < a.m) P[(int64_t)row * a.m + col] = acc[i][j][v];
      }
    }
  }
}

// G[i][j] += sum_s P[s][i][j] for every (i, j) of an upper tile pair; mirrored into the lower triangle.
__global__ __launch_bounds__(256) void gram_reduce(const float* __restrict__ P, int S, int m, float* __restrict__ G,
                                                   int64_t ldg) {
  int bi, bj;
  decode_tile(blockIdx.x, bi, bj);
  const int row0 = bi * TM, col0 = bj * TM;
  const int r = row0 + blockIdx.y * 4 + (threadIdx.x >> 6);
  if (r >= m) return;
  for (int c = col0 + (threadIdx.x & 63); c < min(m, col0 + TM); c += 64) {
    if (bi == bj && c < r) continue;
    float s = 0.f;
    for (int p = 0; p < S; ++p) s += P[((int64_t)p * m + r) * m + c];
    G[(int64_t)r * ldg + c] += s;
    if (c != r) G[(int64_t)c * ldg + r] += s;
  }
}

}  // namespace

extern "C" slim_status slim_hessian_accumulate(slim_ctx* ctx, const void* X, slim_dtype x_dtype, int m, int64_t t_c,
                                               int64_t ldx, float* G, int64_t ldg, int64_t* n_tokens) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, X && G && n_tokens, "slim_hessian_accumulate: null pointer");
  SLIM_REQUIRE(ctx, m > 0 && t_c > 0, "slim_hessian_accumulate: need m > 0 and t_c > 0");
  SLIM_REQUIRE(ctx, m % 8 == 0, "slim_hessian_accumulate: m must be a multiple of 8 (got %d)", m);
  SLIM_REQUIRE(ctx, ldx >= t_c && ldx % 8 == 0, "slim_hessian_accumulate: ldx must be >= t_c and a multiple of 8");
  SLIM_REQUIRE(ctx, ldg >= m, "slim_hessian_accumulate: ldg < m");
  SLIM_REQUIRE(ctx, slim_aligned16(X) && slim_aligned16(G), "slim_hessian_accumulate: misaligned pointer");
  if (x_dtype != SLIM_F16 && x_dtype != SLIM_BF16)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_hessian_accumulate: X must be F16 or BF16");

  const int nt = slim_cdiv(m, TM);
  const int tiles = nt * (nt + 1) / 2;
  const int64_t iters = (t_c + BK - 1) / BK;
  int S = 8;
  while ((int64_t)tiles * S < 1024 && (int64_t)S * 2 * 4 <= iters) S *= 2;
  if (S > iters) S = (int)iters;
  const int64_t kchunk = ((iters + S - 1) / S) * BK;
  S = (int)((t_c + kchunk - 1) / kchunk);

  const size_t pbytes = sizeof(float) * (size_t)S * m * m;
  slim_status st = slim_ws_reserve(ctx, slim_ws_round(pbytes));
  if (st != SLIM_OK) return st;
  GramArgs a;
  a.X = static_cast<const uint16_t*>(X);
  a.ldx = ldx;
  a.m = m;
  a.t = t_c;
  a.kchunk = kchunk;
  a.S = S;
  a.P = static_cast<float*>(slim_ws_alloc(ctx, pbytes));

  static bool attr_done = false;
  if (!attr_done) {
    SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gram_kernel<false>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmemBytes));
    SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gram_kernel<true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmemBytes));
    attr_done = true;
  }
  if (x_dtype == SLIM_BF16)
    SLIM_LAUNCH(ctx, "gram_mfma_bf16", gram_kernel<true>, dim3(tiles * S), dim3(NTHREADS), kSmemBytes, a);
  else
    SLIM_LAUNCH(ctx, "gram_mfma_f16", gram_kernel<false>, dim3(tiles * S), dim3(NTHREADS), kSmemBytes, a);
  SLIM_LAUNCH(ctx, "gram_reduce", gram_reduce, dim3(tiles, TM / 4), dim3(256), 0, a.P, S, m, G, ldg);
  *n_tokens += t_c;
  return SLIM_OK;
}
