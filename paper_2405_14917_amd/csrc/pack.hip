// a9  Storage format (App. B.2): running row offsets of the groups (the cumulative sum that gives every
// group its start row in the packed matrix), the 2-bit-per-group width array, and the bit-packing of the
// codes.  Integer work only; bound by HBM traffic (1 byte read per weight, N/8 bytes written).
//
// pack_codes: one workgroup per (group, slab of 256 output rows).  The slab's 256 x beta codes are read
// with coalesced row accesses into LDS (four codes per word); then thread i of the slab assembles the words of
// output row i one by one, so that the 256 threads write 256 consecutive words of one row of the packed matrix.
#include "slim_internal.h"

namespace {

constexpr int PACK_ROWS = 256;

// single workgroup: validates widths, exclusive scan of beta * b_g / 32, width array
__global__ __launch_bounds__(256) void pack_scan(const uint8_t* __restrict__ bits, int k, int beta, int bit_base,
                                                 int32_t* __restrict__ row_off, uint32_t* __restrict__ gbits,
                                                 int* __restrict__ flags) {
  __shared__ int32_t part[256];
  const int tid = threadIdx.x;
  const int per = (k + 255) / 256;
  const int g0 = tid * per, g1 = min(k, g0 + per);
  int32_t s = 0;
  int bad = 0;
  for (int g = g0; g < g1; ++g) {
    const int b = bits[g];
    if (b < bit_base || b > bit_base + 3 || b > 8 || (beta * b) % 32 != 0) bad = 1;
    s += beta * b / 32;
  }
  part[tid] = s;
  if (tid == 0) flags[0] = 0;
  __syncthreads();
  if (bad) atomicOr(&flags[0], 1);
  // serial prefix over 256 partial sums by every thread for its own start (k is small)
  int32_t base = 0;
  for (int t = 0; t < tid; ++t) base += part[t];
  for (int g = g0; g < g1; ++g) {
    row_off[g] = base;
    base += beta * bits[g] / 32;
  }
  if (g1 == k && g0 < k) row_off[k] = base;
  if (k == 0 && tid == 0) row_off[0] = 0;
  const int nw = (k + 15) / 16;
  for (int w = tid; w < nw; w += 256) {
    uint32_t v = 0;
    for (int j = 0; j < 16 && w * 16 + j < k; ++j) v |= (uint32_t)((bits[w * 16 + j] - bit_base) & 3) << (2 * j);
    gbits[w] = v;
  }
}

__global__ __launch_bounds__(PACK_ROWS) void pack_codes(const uint8_t* __restrict__ codes, int n, int64_t ldc,
                                                        const uint8_t* __restrict__ bits, int beta,
                                                        const int32_t* __restrict__ row_off,
                                                        uint32_t* __restrict__ packed, int64_t packed_rows) {
  extern __shared__ uint32_t tile[];   // [PACK_ROWS][beta / 4 + 1] words of four codes each
  const int g = blockIdx.y;
  const int i0 = blockIdx.x * PACK_ROWS;
  const int rows = min(PACK_ROWS, n - i0);
  const int quads = beta / 4;          // beta is a multiple of 32
  const int stride = quads + 1;        // odd: the rows' words fall into different banks
  const int b = bits[g];
  if (b < 1 || b > 8) return;
  // the slab's codes, sixteen per thread and step where the alignment allows (rows read in whole, coalesced),
  // eight loads in flight per thread
  const uint8_t* src = codes + (int64_t)i0 * ldc + (int64_t)g * beta;
  if ((ldc & 15) == 0 && (reinterpret_cast<uintptr_t>(codes) & 15u) == 0) {
    const int chunks = beta / 16, total = rows * chunks;
    for (int base = 0; base < total; base += 8 * PACK_ROWS) {
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int idx = min(base + u * PACK_ROWS + (int)threadIdx.x, total - 1);
        const int r = idx / chunks, ch = idx - r * chunks;
        v[u] = *reinterpret_cast<const uint4*>(src + (int64_t)r * ldc + 16 * ch);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int idx = base + u * PACK_ROWS + (int)threadIdx.x;
        if (idx < total) {
          const int r = idx / chunks, ch = idx - r * chunks;
          uint32_t* t = tile + r * stride + 4 * ch;
          t[0] = v[u].x, t[1] = v[u].y, t[2] = v[u].z, t[3] = v[u].w;
        }
      }
    }
  } else {
    for (int idx = threadIdx.x; idx < rows * quads; idx += PACK_ROWS) {
      const int r = idx / quads, q = idx - r * quads;
      tile[r * stride + q] = *reinterpret_cast<const uint32_t*>(src + (int64_t)r * ldc + 4 * q);
    }
  }
  __syncthreads();
  const int i = threadIdx.x;
  if (i >= rows) return;
  // Thread i builds the bit stream of output row i0 + i: codes enter a 64-bit window from above, a word leaves it
  // from below whenever 32 bits are complete (element r at bits [r b, (r + 1) b) of the stream, little endian).
  const uint32_t* c = tile + i * stride;
  const uint32_t mask = (1u << b) - 1u;
  uint64_t win = 0;
  int have = 0;
  int64_t r = row_off[g];
  uint32_t* out = packed + i0 + i;
  // four codes at a time: the four bytes of a word are squeezed to 4 b adjacent bits in two steps (bytes to
  // pairs, pairs to the quad), which costs the same for every width
  const uint32_t byte_mask = mask * 0x01010101u;
  for (int q = 0; q < quads; ++q) {
    const uint32_t v = c[q] & byte_mask;
    const uint32_t pair = (v & 0x00ff00ffu) | (((v >> 8) & 0x00ff00ffu) << b);      // codes (0,1) and (2,3), 2 b bits each
    const uint32_t x = (pair & 0xffffu) | ((pair >> 16) << (2 * b));                 // all four, 4 b bits
    win |= (uint64_t)x << have;
    have += 4 * b;
    if (have >= 32) {
      if (r < packed_rows) out[r * n] = (uint32_t)win;
      ++r;
      win >>= 32;
      have -= 32;
    }
  }
}

// Zero points packed with one width along the output channels (App. B.2): word w of group g covers bits
// [32 w, 32 w + 32) of the group's stream, element i (value 2 z_ig) at bits [i zbits, (i + 1) zbits).
// Thread -> (group, word), groups fastest so that the zeros of one output channel are read side by side.
__global__ __launch_bounds__(256) void pack_zeros_kernel(const double* __restrict__ zero, int n, int k, int64_t ldz,
                                                         int zbits, uint32_t* __restrict__ zp, int64_t ldzp, int nw,
                                                         int* __restrict__ n_bad) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)nw * k) return;
  const int g = (int)(idx % k), w = (int)(idx / k);
  const int top = (1 << zbits) - 1;
  const int e0 = (32 * w) / zbits;
  const int e1 = min(n, (32 * w + 32 + zbits - 1) / zbits);
  uint32_t word = 0;
  int bad = 0;
  for (int i = e0; i < e1; ++i) {
    const double u2 = 2.0 * zero[(int64_t)i * ldz + g];
    const double ur = rint(u2);
    int u = (ur < 0.0) ? 0 : ((ur > (double)top) ? top : (int)ur);
    // an element that straddles two words is judged by the word that holds its first bit
    if ((ur != u2 || ur < 0.0 || ur > (double)top) && i * zbits >= 32 * w) ++bad;
    const int sh = i * zbits - 32 * w;
    word |= (sh >= 0) ? ((uint32_t)u << sh) : ((uint32_t)u >> (-sh));
  }
  zp[(int64_t)g * ldzp + w] = word;
  if (bad) atomicAdd(n_bad, bad);
}

__global__ __launch_bounds__(256) void unpack_zeros_kernel(const uint32_t* __restrict__ zp, int64_t ldzp, int n, int k,
                                                           int zbits, double* __restrict__ zero, int64_t ldz) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)n * k) return;
  const int g = (int)(idx % k), i = (int)(idx / k);
  const int bit = i * zbits, w = bit / 32, sh = bit % 32;
  uint64_t two = zp[(int64_t)g * ldzp + w];
  if (sh + zbits > 32) two |= (uint64_t)zp[(int64_t)g * ldzp + w + 1] << 32;
  zero[(int64_t)i * ldz + g] = 0.5 * (double)((two >> sh) & ((1u << zbits) - 1u));
}

__global__ void clear_flag(int* f) { *f = 0; }

}  // namespace

extern "C" slim_status slim_pack_zeros(slim_ctx* ctx, const double* zero, int n, int k, int64_t ldz, int zbits,
                                       uint32_t* zpacked, int64_t ldzp, int* n_bad) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, zero && zpacked, "slim_pack_zeros: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && k > 0 && ldz >= k, "slim_pack_zeros: need n, k > 0 and ldz >= k");
  SLIM_REQUIRE(ctx, zbits >= 2 && zbits <= 16, "slim_pack_zeros: zbits must be in 2..16 (got %d)", zbits);
  const int nw = slim_cdiv((int64_t)n * zbits, 32);
  SLIM_REQUIRE(ctx, ldzp >= nw, "slim_pack_zeros: ldzp must be at least ceil(n zbits / 32) = %d", nw);
  int* flag = ctx->dflags + 2;
  SLIM_LAUNCH(ctx, "pack_zeros_clear", clear_flag, dim3(1), dim3(1), 0, flag);
  SLIM_LAUNCH(ctx, "pack_zeros", pack_zeros_kernel, dim3(slim_cdiv((int64_t)nw * k, 256)), dim3(256), 0, zero, n, k, ldz,
              zbits, zpacked, ldzp, nw, flag);
  if (!n_bad) return SLIM_OK;                      // nothing for the host: the call does not wait
  int* host = reinterpret_cast<int*>(ctx->hpin);
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(host, flag, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  *n_bad = host[0];
  return SLIM_OK;
}

extern "C" slim_status slim_unpack_zeros(slim_ctx* ctx, const uint32_t* zpacked, int64_t ldzp, int n, int k, int zbits,
                                         double* zero, int64_t ldz) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, zero && zpacked, "slim_unpack_zeros: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && k > 0 && ldz >= k, "slim_unpack_zeros: need n, k > 0 and ldz >= k");
  SLIM_REQUIRE(ctx, zbits >= 2 && zbits <= 16, "slim_unpack_zeros: zbits must be in 2..16 (got %d)", zbits);
  SLIM_REQUIRE(ctx, ldzp >= slim_cdiv((int64_t)n * zbits, 32), "slim_unpack_zeros: ldzp too small");
  SLIM_LAUNCH(ctx, "unpack_zeros", unpack_zeros_kernel, dim3(slim_cdiv((int64_t)n * k, 256)), dim3(256), 0, zpacked, ldzp,
              n, k, zbits, zero, ldz);
  return SLIM_OK;
}

extern "C" slim_status slim_pack(slim_ctx* ctx, const uint8_t* codes, int n, int m, int64_t ldc, const uint8_t* bits,
                                 int beta, int bit_base, uint32_t* packed, int64_t packed_rows, uint32_t* gbits,
                                 int32_t* row_off, int* m_star) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, codes && bits && packed && gbits && row_off, "slim_pack: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "slim_pack: need n, m > 0 and beta | m");
  SLIM_REQUIRE(ctx, beta % 32 == 0, "slim_pack: beta must be a multiple of 32 (got %d)", beta);
  SLIM_REQUIRE(ctx, ldc >= m && ldc % 4 == 0 && (reinterpret_cast<uintptr_t>(codes) & 3u) == 0,
               "slim_pack: codes must be 4-byte aligned with ldc a multiple of 4");
  SLIM_REQUIRE(ctx, packed_rows >= 0, "slim_pack: negative capacity");
  SLIM_REQUIRE(ctx, bit_base >= 1 && bit_base <= 5, "slim_pack: bit_base must be in 1..5 (got %d)", bit_base);
  const int k = m / beta;
  int* flags = ctx->dflags;   // flags[0] is cleared by pack_scan itself
  SLIM_LAUNCH(ctx, "pack_scan", pack_scan, dim3(1), dim3(256), 0, bits, k, beta, bit_base, row_off, gbits, flags);
  const size_t smem = sizeof(uint32_t) * (size_t)PACK_ROWS * (beta / 4 + 1);
  if (smem > 160 * 1024) return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "slim_pack: beta = %d is too large (at most 636)", beta);
  if (smem > 64 * 1024) {
    static bool done = false;
    if (!done) {
      SLIM_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(pack_codes),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
      done = true;
    }
  }
  SLIM_LAUNCH(ctx, "pack_codes", pack_codes, dim3(slim_cdiv(n, PACK_ROWS), k), dim3(PACK_ROWS), smem, codes, n, ldc,
              bits, beta, row_off, packed, packed_rows);
  if (!m_star) return SLIM_OK;                     // nothing for the host: the call does not wait (and cannot report)
  int* host = reinterpret_cast<int*>(ctx->hpin);
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(&host[0], row_off + k, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipMemcpyAsync(&host[1], flags, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
  SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  *m_star = host[0];
  if (host[1] != 0)
    return slim_fail(ctx, SLIM_ERR_INVALID_ARG, "slim_pack: a width is outside bit_base .. bit_base + 3 (%d .. %d, at most 8) or beta * width is not a multiple of 32",
                     bit_base, bit_base + 3);
  if (host[0] > packed_rows)
    return slim_fail(ctx, SLIM_ERR_INVALID_ARG, "slim_pack: packed needs %d rows, capacity is %lld", host[0],
                     (long long)packed_rows);
  return SLIM_OK;
}
