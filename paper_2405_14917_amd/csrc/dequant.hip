// The linear layer on the stored form (App. B.2, inference): Y = X dequant(W_int)^T straight from the packed
// integers, the group-width array and the start rows that slim_pack writes, with the scales and zeros of
// slim_gptq_quantize.  W^_ij = scale[i][g] (q_ij - zero[i][g]), g = j / beta (Eq. 1).
//
// For the few tokens of a decoding step the layer is a stream over the packed weights: 2 bits per weight on
// average, read once.  A thread owns one output row i (one column of W_int, so that the 256 threads of a
// workgroup read 1 KiB of consecutive words per step), walks a range of groups and dequantises a group's bit
// stream 32 elements at a time; the group's activations sit in LDS and are read by all threads at once
// (broadcast).  Several workgroups share a block of output rows by splitting the groups among them; their
// partial sums are added in a fixed order by a second kernel, so the result does not depend on timing.
//
// The paper's kernel (an extension of AutoGPTQ's, for 32-wide warps) has the same division of labour - a thread
// dequantises a contiguous segment of one column and dots it with activations shared in the block; what differs
// is the mapping to 64-wide wavefronts, the LDS broadcast, and the deterministic two-stage reduction in place of
// atomics.
#include <algorithm>

#include "slim_device.h"
#include "slim_internal.h"

namespace {

using namespace slimdev;

constexpr int DQ_THREADS = 256;
constexpr int DQ_MAX_T = 16;

struct DqArgs {
  const uint32_t* packed;
  int64_t ldp;
  const uint32_t* gbits;
  const int32_t* row_off;
  const double* scale;   // n x k
  const double* zero;    // n x k
  int n, m, beta, k;
  const void* X;         // t_x x m, 16-bit
  int x_bf16;
  int t_x;
  int64_t ldx;
  int gper;              // groups per workgroup along grid.y
  float* out;            // Y (one split) or the partial sums [split][T][n]
  int64_t ldo;           // leading dimension of `out` per token
  int64_t split_stride;  // elements between the partial sums of two splits (0 when writing Y)
};

__device__ __forceinline__ float widen16(uint16_t h, int bf16) {
  if (bf16) return __uint_as_float((unsigned)h << 16);
  return __half2float(__ushort_as_half(h));
}

// acc[t] += (q - z) x[t][r0 + e] for the 32 elements e of one chunk of a group's bit stream; `w` holds its B words.
template <int B, int T>
__device__ __forceinline__ void chunk_dot(const uint32_t (&w)[B], float z, const float* __restrict__ xs, int beta,
                                          int r0, float (&acc)[T]) {
  auto use = [&](int e, unsigned q) {
    const float d = (float)q - z;
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = fmaf(d, xs[t * beta + r0 + e], acc[t]);
  };
  if (B == 3) {
    // 96 bits: elements 0 .. 20 lie in the first 63, element 21 starts at bit 63
    const uint64_t lo = (uint64_t)w[0] | ((uint64_t)w[1 % B] << 32);
    const uint64_t hi = ((uint64_t)w[2 % B] << 1) | (w[1 % B] >> 31);
#pragma unroll
    for (int e = 0; e < 21; ++e) use(e, (unsigned)(lo >> (3 * e)) & 7u);
#pragma unroll
    for (int e = 21; e < 32; ++e) use(e, (unsigned)(hi >> (3 * (e - 21))) & 7u);
  } else {
    constexpr int PER = 32 / B;            // elements per word: no element straddles two words
#pragma unroll
    for (int wi = 0; wi < B; ++wi)
#pragma unroll
      for (int e = 0; e < PER; ++e) use(wi * PER + e, (w[wi] >> (B * e)) & ((1u << B) - 1u));
  }
}

template <int B, int T>
__device__ __forceinline__ void group_dot(const DqArgs& a, int i, int base, float z, const float* xs, float (&acc)[T]) {
  const uint32_t* p = a.packed + (int64_t)base * a.ldp + i;
  for (int c = 0; c < a.beta / 32; ++c) {
    uint32_t w[B];
#pragma unroll
    for (int wi = 0; wi < B; ++wi) w[wi] = p[(int64_t)(c * B + wi) * a.ldp];
    chunk_dot<B, T>(w, z, xs, a.beta, 32 * c, acc);
  }
}

template <int T>
__global__ __launch_bounds__(DQ_THREADS) void dequant_matmul(DqArgs a) {
  extern __shared__ float xs[];                    // [T][beta]: the current group's activations
  const int tid = threadIdx.x;
  const int i = blockIdx.x * DQ_THREADS + tid;     // output row
  const int g0 = blockIdx.y * a.gper, g1 = min(a.k, g0 + a.gper);
  float y[T];
#pragma unroll
  for (int t = 0; t < T; ++t) y[t] = 0.f;
  const uint16_t* X = static_cast<const uint16_t*>(a.X);
  for (int g = g0; g < g1; ++g) {
    __syncthreads();
    for (int idx = tid; idx < T * a.beta; idx += DQ_THREADS) {
      const int t = idx / a.beta, r = idx - t * a.beta;
      xs[idx] = (t < a.t_x) ? widen16(X[(int64_t)t * a.ldx + (int64_t)g * a.beta + r], a.x_bf16) : 0.f;
    }
    __syncthreads();
    if (i < a.n) {
      const int b = (int)((a.gbits[g >> 4] >> (2 * (g & 15))) & 3u) + 1;
      const int base = a.row_off[g];
      const float s = (float)a.scale[(int64_t)i * a.k + g], z = (float)a.zero[(int64_t)i * a.k + g];
      float acc[T];
#pragma unroll
      for (int t = 0; t < T; ++t) acc[t] = 0.f;
      switch (b) {                                 // the same for the whole workgroup
        case 1: group_dot<1, T>(a, i, base, z, xs, acc); break;
        case 2: group_dot<2, T>(a, i, base, z, xs, acc); break;
        case 3: group_dot<3, T>(a, i, base, z, xs, acc); break;
        default: group_dot<4, T>(a, i, base, z, xs, acc); break;
      }
#pragma unroll
      for (int t = 0; t < T; ++t) y[t] = fmaf(s, acc[t], y[t]);
    }
  }
  if (i < a.n) {
    float* o = a.out + (int64_t)blockIdx.y * a.split_stride;
#pragma unroll
    for (int t = 0; t < T; ++t)
      if (t < a.t_x) o[(int64_t)t * a.ldo + i] = y[t];
  }
}

// Y[t][i] = sum over the splits, in split order
__global__ __launch_bounds__(256) void dequant_reduce(const float* __restrict__ part, int splits, int64_t split_stride,
                                                      int t_x, int n, float* __restrict__ Y, int64_t ldy) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)t_x * n) return;
  const int t = (int)(idx / n), i = (int)(idx - (int64_t)t * n);
  float s = 0.f;
  for (int p = 0; p < splits; ++p) s += part[p * split_stride + (int64_t)t * n + i];
  Y[(int64_t)t * ldy + i] = s;
}

template <int T>
slim_status launch(slim_ctx* ctx, const DqArgs& a, dim3 grid, size_t smem) {
  SLIM_LAUNCH(ctx, "dequant_matmul", dequant_matmul<T>, grid, dim3(DQ_THREADS), smem, a);
  return SLIM_OK;
}

}  // namespace

extern "C" slim_status slim_dequant_matmul(slim_ctx* ctx, const uint32_t* packed, int64_t ldp, const uint32_t* gbits,
                                           const int32_t* row_off, const double* scale, const double* zero, int n,
                                           int m, int beta, const void* X, slim_dtype x_dtype, int t_x, int64_t ldx,
                                           float* Y, int64_t ldy) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, packed && gbits && row_off && scale && zero && X && Y, "slim_dequant_matmul: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "slim_dequant_matmul: need n, m > 0 and beta | m");
  SLIM_REQUIRE(ctx, beta % 32 == 0, "slim_dequant_matmul: beta must be a multiple of 32 (got %d)", beta);
  SLIM_REQUIRE(ctx, t_x >= 1 && t_x <= DQ_MAX_T, "slim_dequant_matmul: t_x must be in 1..%d (got %d)", DQ_MAX_T, t_x);
  SLIM_REQUIRE(ctx, ldp >= n && ldx >= m && ldy >= n, "slim_dequant_matmul: leading dimension too small");
  if (x_dtype != SLIM_F16 && x_dtype != SLIM_BF16)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_dequant_matmul: X must be F16 or BF16");
  const int k = m / beta;
  int T = 1;
  while (T < t_x) T *= 2;
  const size_t smem = sizeof(float) * (size_t)T * beta;
  const int gx = slim_cdiv(n, DQ_THREADS);
  // enough workgroups to fill the chip twice over, by splitting the groups
  const int cus = std::max(1, ctx->num_cus);
  const int splits_wanted = std::max(1, std::min(k, (2 * cus + gx - 1) / gx));
  const int gper = slim_cdiv(k, splits_wanted);
  const int splits = slim_cdiv(k, gper);

  DqArgs a;
  a.packed = packed;
  a.ldp = ldp;
  a.gbits = gbits;
  a.row_off = row_off;
  a.scale = scale;
  a.zero = zero;
  a.n = n;
  a.m = m;
  a.beta = beta;
  a.k = k;
  a.X = X;
  a.x_bf16 = (x_dtype == SLIM_BF16);
  a.t_x = t_x;
  a.ldx = ldx;
  a.gper = gper;
  float* part = nullptr;
  if (splits > 1) {
    slim_status st = slim_ws_reserve(ctx, slim_ws_round(sizeof(float) * (size_t)splits * t_x * n));
    if (st != SLIM_OK) return st;
    part = static_cast<float*>(slim_ws_alloc(ctx, sizeof(float) * (size_t)splits * t_x * n));
    a.out = part;
    a.ldo = n;
    a.split_stride = (int64_t)t_x * n;
  } else {
    a.out = Y;
    a.ldo = ldy;
    a.split_stride = 0;
  }
  const dim3 grid(gx, splits);
  slim_status st;
  switch (T) {
    case 1: st = launch<1>(ctx, a, grid, smem); break;
    case 2: st = launch<2>(ctx, a, grid, smem); break;
    case 4: st = launch<4>(ctx, a, grid, smem); break;
    case 8: st = launch<8>(ctx, a, grid, smem); break;
    default: st = launch<16>(ctx, a, grid, smem); break;
  }
  if (st != SLIM_OK) return st;
  if (splits > 1)
    SLIM_LAUNCH(ctx, "dequant_reduce", dequant_reduce, dim3(slim_cdiv((int64_t)t_x * n, 256)), dim3(256), 0, part, splits,
                a.split_stride, t_x, n, Y, ldy);
  return SLIM_OK;
}
