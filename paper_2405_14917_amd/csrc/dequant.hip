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

#include <mutex>

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
  int bit_base;          // the width that the 2-bit group value 0 stands for
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
  } else if (32 % B != 0) {
    // any other width that does not divide 32 (5: 160 bits in 5 words): an element that straddles takes its upper
    // bits from the next word; every index and shift is a compile-time constant after unrolling
#pragma unroll
    for (int e = 0; e < 32; ++e) {
      const int wi = (e * B) / 32, sh = (e * B) % 32;
      unsigned v = w[wi] >> sh;
      if (sh + B > 32) v |= w[(wi + 1) % B] << (32 - sh);
      use(e, v & ((1u << B) - 1u));
    }
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
      const int b = (int)((a.gbits[g >> 4] >> (2 * (g & 15))) & 3u) + a.bit_base;
      const int base = a.row_off[g];
      // a group whose start rows disagree with its width (a stored form read with the wrong bit_base, or a damaged
      // one) is skipped: its words are never touched, so no read leaves the rows the stored form itself declares
      if ((a.row_off[g + 1] - base) * 32 != a.beta * b) continue;
      const float s = (float)a.scale[(int64_t)i * a.k + g], z = (float)a.zero[(int64_t)i * a.k + g];
      float acc[T];
#pragma unroll
      for (int t = 0; t < T; ++t) acc[t] = 0.f;
      switch (b) {                                 // the same for the whole workgroup
        case 1: group_dot<1, T>(a, i, base, z, xs, acc); break;
        case 2: group_dot<2, T>(a, i, base, z, xs, acc); break;
        case 3: group_dot<3, T>(a, i, base, z, xs, acc); break;
        case 4: group_dot<4, T>(a, i, base, z, xs, acc); break;
        default: group_dot<5, T>(a, i, base, z, xs, acc); break;
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

// ------------------------------------------------------------------------------------------------------
// The same product on the matrix cores, for fp16 activations.  v_mfma_f32_32x32x16_f16 with the tokens as rows
// of the first operand and the output rows of the layer as columns of the second: a lane then owns ONE output
// row (its scale and zero are lane constants) and the 16 tokens of its accumulator registers.  The second
// operand is 2 (q - z), formed exactly in fp16 from the packed codes without any conversion instruction: a code
// q shifted left by one and OR-ed into the mantissa of 1024.0 is the fp16 number 1024 + 2 q, and subtracting
// 1024 + 2 z (2 z is an integer: zeros are integers, or 1/2 for the sign form of width 1; other zeros: see below) leaves 2 (q - z);
// the factor 1/2 goes into the scale.  Two codes are handled per instruction (packed fp16): the eight codes a
// lane needs for one MFMA are first spread so that code j sits in the low and code j + 4 in the high half of a
// register, and the activations are stored in LDS in that order (0 4 1 5 2 6 3 7) to match.  Products are exact
// (11-bit by 6-bit), the sums are fp32 in the matrix core, the scale is applied per group in fp32.
// With up to 32 tokens served by the same instructions, the kernel is a stream over the packed weights.
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int DM_WAVES = 4, DM_ROWS = 32 * DM_WAVES, DM_TOK = 32, DM_PAD = 8;

// the 8 B-bit codes in the low bits of v -> four registers of packed fp16 pairs (1024 + 2 c_j, 1024 + 2 c_{j+4})
template <int B>
__device__ __forceinline__ void spread_codes(unsigned v, unsigned (&t)[4]) {
  constexpr unsigned M2 = ((1u << B) - 1u) << 1;
  const unsigned u = (B == 4) ? v : ((v & ((1u << (4 * B)) - 1u)) | ((v >> (4 * B)) << 16));
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const unsigned sh = (B * j >= 1) ? (u >> (B * j - 1)) : (u << 1);
    t[j] = (sh & (M2 | (M2 << 16))) | 0x64006400u;
  }
}

// the same for codes wider than 4 bits: the 8 codes take 8 B > 32 bits
template <int B>
__device__ __forceinline__ void spread_codes_wide(uint64_t v, unsigned (&t)[4]) {
  constexpr unsigned M = (1u << B) - 1u;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    t[j] = (((unsigned)(v >> (B * j)) & M) << 1) | (((unsigned)(v >> (B * (j + 4))) & M) << 17) | 0x64006400u;
}

// One sub-block of SUB codes (SUB / 16 MFMA steps) of one group: `w` holds the SUB * B / 32 words of the lane's
// output row; xs points at the lane's token row of the activation tile, at this sub-block's first column.
template <int B, int SUB, int MAXW>
__device__ __forceinline__ float16v subblock_mfma(const unsigned (&w)[MAXW], int h, half2v zz, const _Float16* xs,
                                                  float16v acc) {
  constexpr int NW = SUB * B / 32;
  static_assert(NW <= MAXW, "the sub-block's words do not fit the register array");
#pragma unroll
  for (int st = 0; st < SUB / 16; ++st) {
    unsigned t[4];
    if constexpr (B > 4) {
      // 8 codes = 8 B bits (at most 64) starting at bit 8 B (2 st + h): always within two consecutive words for
      // B = 5 (the start is a multiple of 8, so at most 24 + 40 bits)
      static_assert(B == 5, "wider codes would span three words");
      auto unit_wide = [&](int unit) -> uint64_t {
        const int bit = 8 * B * unit, wi = bit / 32, sh = bit % 32;
        const uint64_t two = (uint64_t)w[wi] | ((uint64_t)w[(wi + 1 < NW) ? wi + 1 : wi] << 32);
        return two >> sh;
      };
      const uint64_t v0 = unit_wide(2 * st), v1 = unit_wide(2 * st + 1);
      spread_codes_wide<B>(h ? v1 : v0, t);
    } else {
    // unit 2 st + h of the stream: 8 codes = 8 B bits starting at bit 8 B (2 st + h)
    auto unit_bits = [&](int unit) -> unsigned {
      const int bit = 8 * B * unit, wi = bit / 32, sh = bit % 32;
      if (sh + 8 * B <= 32) return w[wi] >> sh;
      const uint64_t two = (uint64_t)w[wi] | ((uint64_t)w[(wi + 1 < NW) ? wi + 1 : wi] << 32);
      return (unsigned)(two >> sh);
    };
    const unsigned v0 = unit_bits(2 * st), v1 = unit_bits(2 * st + 1);   // the unit for h = 0 and for h = 1
    spread_codes<B>(h ? v1 : v0, t);
    }
    half8v bfrag;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const half2v d = *reinterpret_cast<const half2v*>(&t[j]) - zz;
      bfrag[2 * j] = d[0];
      bfrag[2 * j + 1] = d[1];
    }
    const half8v afrag = *reinterpret_cast<const half8v*>(xs + 16 * st + 8 * h);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(afrag, bfrag, acc, 0, 0, 0);
  }
  return acc;
}

// SUB = min(beta, 128): a group is worked off in beta / SUB sub-blocks.  The activations of the workgroup's whole
// group range are put into LDS once (rows of the real tokens plus one row of zeros that the lanes of the other
// token slots read); the words, scale and zero of the next sub-block are fetched while the current one is
// multiplied, so that a workgroup waits for memory once, not once per group.
// MAXW: words of a sub-block at the widest width in the layer (16 for widths up to 4, 20 with five-bit groups).
template <int SUB, int MAXW>
__global__ __launch_bounds__(64 * DM_WAVES) void dequant_matmul_mfma(DqArgs a) {
  extern __shared__ __align__(16) _Float16 xh[];   // [t_x + 1][cols + DM_PAD], every 8 columns in the order 0 4 1 5 2 6 3 7
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int row = min(blockIdx.x * DM_ROWS + wave * 32 + l32, a.n - 1);    // clamped: rows past the end are not stored
  const int g0 = blockIdx.y * a.gper, g1 = min(a.k, g0 + a.gper);
  const int cols = (g1 - g0) * a.beta, ldxs = cols + DM_PAD;
  const uint16_t* X = static_cast<const uint16_t*>(a.X);
  for (int idx = tid; idx < (a.t_x + 1) * (cols / 8); idx += 64 * DM_WAVES) {
    const int t = idx / (cols / 8), c = idx - t * (cols / 8);
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (t < a.t_x) raw = *reinterpret_cast<const uint4*>(X + (int64_t)t * a.ldx + (int64_t)g0 * a.beta + 8 * c);
    // halves 0..7 of the chunk are (raw.x lo, hi), (raw.y lo, hi), ...; stored as 0 4 1 5 2 6 3 7
    uint4 o;
    o.x = (raw.x & 0xffffu) | (raw.z << 16);
    o.y = (raw.x >> 16) | (raw.z & 0xffff0000u);
    o.z = (raw.y & 0xffffu) | (raw.w << 16);
    o.w = (raw.y >> 16) | (raw.w & 0xffff0000u);
    *reinterpret_cast<uint4*>(xh + t * ldxs + 8 * c) = o;
  }
  const _Float16* xs = xh + min(l32, a.t_x) * ldxs;
  // The scales (halved: the codes are doubled) and the zeros (as 1024 + 2 z in fp16) of the workgroup's rows and
  // groups, fetched together: per (row, group) loads by the lane that owns the row would touch 32 cache lines per
  // instruction, eight times the requests of the packed words themselves.
  const int gcount = g1 - g0;
  // A zero outside that form (Eq. 1 puts no bound on -round(w_min / delta0): a group of one sign with a narrow
  // range has a large one) is split: z0, the nearest value that has the form, goes through the matrix cores, and
  // the rest enters as  - 2 (z - z0) sum_j x_j  when the group is complete (zr != 0, rare).
  float* sp = reinterpret_cast<float*>(xh + (a.t_x + 1) * ldxs);            // [DM_ROWS][gcount]
  float* zr = sp + DM_ROWS * gcount;                                          // [DM_ROWS][gcount]
  _Float16* zp = reinterpret_cast<_Float16*>(zr + DM_ROWS * gcount);          // [DM_ROWS][gcount]
  for (int idx = tid; idx < DM_ROWS * gcount; idx += 64 * DM_WAVES) {
    const int r = idx / gcount, gi = idx - r * gcount;
    const int64_t src = (int64_t)min(blockIdx.x * DM_ROWS + r, a.n - 1) * a.k + g0 + gi;
    sp[idx] = (float)(0.5 * a.scale[src]);
    const double z2 = 2.0 * a.zero[src];
    const double z02 = fmin(fmax(rint(z2), -1022.0), 1022.0);
    zp[idx] = (_Float16)(float)(1024.0 + z02);                                // exact: an integer in 2 .. 2046
    zr[idx] = (float)(z2 - z02);
  }
  const int prow = (wave * 32 + l32) * gcount;

  const int nsub = a.beta / SUB, units = (g1 - g0) * nsub;
  auto width = [&](int g) { return (int)((a.gbits[g >> 4] >> (2 * (g & 15))) & 3u) + a.bit_base; };
  // fetch of unit u: the words of the lane's row
  // 0 for a group whose start rows disagree with its width: such a group is skipped and none of its words is read
  auto checked_width = [&](int g) {
    const int b = width(g);
    return ((a.row_off[g + 1] - a.row_off[g]) * 32 == a.beta * b) ? b : 0;
  };
  auto fetch = [&](int u, unsigned (&w)[MAXW]) {
    const int g = g0 + u / nsub, sb = u - (u / nsub) * nsub;
    const int nwu = SUB * checked_width(g) / 32;
    const uint32_t* p = a.packed + (int64_t)(a.row_off[g] + sb * nwu) * a.ldp + row;
#pragma unroll
    for (int i = 0; i < MAXW; ++i) w[i] = (i < nwu) ? p[(int64_t)i * a.ldp] : 0u;
  };
  unsigned wc[MAXW], wn[MAXW];
  fetch(0, wc);
  __syncthreads();                                 // the activation tile and the parameters are complete

  float y[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) y[v] = 0.f;
  float16v acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int u = 0; u < units; ++u) {
    const int g = g0 + u / nsub, sb = u - (u / nsub) * nsub;
    if (u + 1 < units) fetch(u + 1, wn);
    const _Float16 zc = zp[prow + (g - g0)];
    half2v zz;
    zz[0] = zc;
    zz[1] = zc;
    const _Float16* xu = xs + (g - g0) * a.beta + sb * SUB;
    switch (checked_width(g)) {                    // the same for the whole workgroup
      case 0: break;
      case 1: acc = subblock_mfma<1, SUB, MAXW>(wc, h, zz, xu, acc); break;
      case 2: acc = subblock_mfma<2, SUB, MAXW>(wc, h, zz, xu, acc); break;
      case 3: acc = subblock_mfma<3, SUB, MAXW>(wc, h, zz, xu, acc); break;
      case 4: acc = subblock_mfma<4, SUB, MAXW>(wc, h, zz, xu, acc); break;
      default:
        if constexpr (MAXW >= 20) acc = subblock_mfma<5, SUB, MAXW>(wc, h, zz, xu, acc);
        break;
    }
    if (sb == nsub - 1) {                          // the group is complete: its scale (times the 1/2 of the doubled codes)
      const float rest = zr[prow + (g - g0)];
      if (__builtin_amdgcn_ballot_w64(rest != 0.f) != 0 && checked_width(g) != 0) {
        // some row of this wavefront has a zero that the fp16 form does not hold: the part it does not hold times
        // the sum of the group's activations, per token (the order of the tile's columns does not matter for a sum)
#pragma unroll 1
        for (int v = 0; v < 16; ++v) {
          const int t = 8 * (v >> 2) + 4 * h + (v & 3);
          const _Float16* xt = xh + min(t, a.t_x) * ldxs + (g - g0) * a.beta;
          float sx = 0.f;
          for (int j = 0; j < a.beta; ++j) sx += (float)xt[j];
          acc[v] = fmaf(-rest, sx, acc[v]);
        }
      }
      const float s2 = sp[prow + (g - g0)];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        y[v] = fmaf(s2, acc[v], y[v]);
        acc[v] = 0.f;
      }
    }
#pragma unroll
    for (int i = 0; i < MAXW; ++i) wc[i] = wn[i];
  }
  if (blockIdx.x * DM_ROWS + wave * 32 + l32 < a.n) {
    float* o = a.out + (int64_t)blockIdx.y * a.split_stride + row;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int t = 8 * (v >> 2) + 4 * h + (v & 3);   // accumulator register v of lane (l32, h): token t, output row l32
      if (t < a.t_x) o[(int64_t)t * a.ldo] = y[v];
    }
  }
}

template <int T>
slim_status launch(slim_ctx* ctx, const DqArgs& a, dim3 grid, size_t smem) {
  SLIM_LAUNCH(ctx, "dequant_matmul@dequant_matmul<T>", dequant_matmul<T>, grid, dim3(DQ_THREADS), smem, a);
  return SLIM_OK;
}

// Partial sums of the group ranges for callers that must not allocate: one array per GPU, held from the moment the
// library's code is loaded on that GPU until the process ends.  Host code never uses the array's name as an
// address; the device address is asked for once per device (slim_dq_scratch_resolve) and kept.
constexpr size_t DQ_SCRATCH_FLOATS = SLIM_DEQUANT_NOALLOC_MAX_FLOATS;      // 16 MiB
static __device__ __align__(256) float scratch[DQ_SCRATCH_FLOATS];

constexpr int DQ_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[DQ_MAX_DEVICES] = {};

// Group ranges the layer is split into (and groups per range), for the matrix-core kernel or the plain one:
// enough workgroups per CU to hide the latency of their loads behind one another; fewer for a small layer, where
// the reduction over the ranges would cost more than the ranges gain.
int dq_splits(int n, int m, int beta, int t_x, int cus, bool mfma, int& gper) {
  const int k = m / beta;
  const bool small = 2 * slim_cdiv(n, DM_ROWS) < cus;
  const int gx = slim_cdiv(n, mfma ? DM_ROWS : DQ_THREADS);
  const int per_cu = small ? 2 : 8;
  const int splits_wanted = std::max(1, std::min(k, (per_cu * cus + gx - 1) / gx));
  gper = slim_cdiv(k, splits_wanted);
  if (mfma) {
    // the activations of a workgroup's group range (t_x + 1 rows of 16-bit values) and its rows' parameters
    // (10 bytes per row and group) have to fit into 64 KiB of LDS
    const int fit = std::max(1, (int)((64 * 1024 - 2 * (t_x + 1) * DM_PAD) / (2 * (t_x + 1) * beta + 10 * DM_ROWS)));
    gper = std::min(gper, fit);
  }
  return slim_cdiv(k, gper);
}

// The whole call.  `fixed` = nullptr: partial sums go to the context's workspace (grown if needed); otherwise to
// `fixed`, which holds `fixed_floats` floats, and nothing is allocated.
slim_status dequant_matmul_run(slim_ctx* ctx, const char* fn, const uint32_t* packed, int64_t ldp,
                               const uint32_t* gbits, const int32_t* row_off, const double* scale, const double* zero,
                               int n, int m, int beta, int bit_base, const void* X, slim_dtype x_dtype, int t_x,
                               int64_t ldx, float* Y, int64_t ldy, float* fixed, size_t fixed_floats) {
  SLIM_REQUIRE(ctx, packed && gbits && row_off && scale && zero && X && Y, "%s: null pointer", fn);
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "%s: need n, m > 0 and beta | m", fn);
  SLIM_REQUIRE(ctx, beta % 32 == 0, "%s: beta must be a multiple of 32 (got %d)", fn, beta);
  SLIM_REQUIRE(ctx, t_x >= 1 && t_x <= DQ_MAX_T, "%s: t_x must be in 1..%d (got %d)", fn, DQ_MAX_T, t_x);
  SLIM_REQUIRE(ctx, ldp >= n && ldx >= m && ldy >= n, "%s: leading dimension too small", fn);
  if (x_dtype != SLIM_F16 && x_dtype != SLIM_BF16)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "%s: X must be F16 or BF16", fn);
  if (bit_base != 1 && bit_base != 2)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "%s: bit_base must be 1 or 2 (widths up to 5), got %d", fn, bit_base);
  const int k = m / beta;
  int T = 1;
  while (T < t_x) T *= 2;
  // fp16 activations that can be fetched 16 bytes at a time go to the matrix-core kernel
  // (a layer too small to give every CU a few workgroups of that kernel is bound by launch and reduction, and
  // for one or two tokens the plain kernel, whose workgroups cover twice the rows, is the quicker one there)
  const int cus = std::max(1, ctx->num_cus);
  const bool small = 2 * slim_cdiv(n, DM_ROWS) < cus;
  const bool mfma = x_dtype == SLIM_F16 && slim_aligned16(X) && ldx % 8 == 0 &&
                    (beta == 32 || beta == 64 || beta % 128 == 0) && !(small && t_x <= 2);
  size_t smem = sizeof(float) * (size_t)T * beta;   // (the matrix-core kernel's depends on the split, below)
  const int gx = slim_cdiv(n, mfma ? DM_ROWS : DQ_THREADS);
  int gper = 0;
  const int splits = dq_splits(n, m, beta, t_x, cus, mfma, gper);

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
  a.bit_base = bit_base;
  a.X = X;
  a.x_bf16 = (x_dtype == SLIM_BF16);
  a.t_x = t_x;
  a.ldx = ldx;
  a.gper = gper;
  float* part = nullptr;
  if (splits > 1) {
    const size_t part_floats = (size_t)splits * t_x * n;
    if (fixed) {
      if (part_floats > fixed_floats)
        return slim_fail(ctx, SLIM_ERR_UNSUPPORTED,
                         "%s: this layer needs %zu floats of partial sums (%d group ranges x %d tokens x %d rows), the "
                         "fixed buffer holds %zu: fewer tokens per call, or slim_dequant_matmul", fn, part_floats,
                         splits, t_x, n, fixed_floats);
      part = fixed;
    } else {
      slim_status st = slim_ws_reserve(ctx, slim_ws_need_dequant(n, m, beta, t_x, cus));
      if (st != SLIM_OK) return st;
      part = static_cast<float*>(slim_ws_alloc(ctx, sizeof(float) * part_floats));
    }
    a.out = part;
    a.ldo = n;
    a.split_stride = (int64_t)t_x * n;
  } else {
    a.out = Y;
    a.ldo = ldy;
    a.split_stride = 0;
  }
  const dim3 grid(gx, splits);
  slim_status st = SLIM_OK;
  if (mfma) {
    smem = sizeof(uint16_t) * (size_t)(t_x + 1) * ((size_t)gper * beta + DM_PAD) + (size_t)DM_ROWS * gper * 10;
#define SLIM_DQ_MFMA(SUB, MAXW)                                                                              \
  SLIM_LAUNCH(ctx, "dequant_matmul@dequant_matmul_mfma<" #SUB ", " #MAXW ">", (dequant_matmul_mfma<SUB, MAXW>), grid, \
              dim3(64 * DM_WAVES), smem, a)
    const bool wide = bit_base + 3 > 4;            // the layer may hold five-bit groups
    if (beta >= 128) {
      if (wide) SLIM_DQ_MFMA(128, 20); else SLIM_DQ_MFMA(128, 16);
    } else if (beta == 64) {
      if (wide) SLIM_DQ_MFMA(64, 20); else SLIM_DQ_MFMA(64, 16);
    } else {
      if (wide) SLIM_DQ_MFMA(32, 20); else SLIM_DQ_MFMA(32, 16);
    }
#undef SLIM_DQ_MFMA
  } else
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

// Any number of tokens: DQ_MAX_T at a time, one after the other on the context's stream (the kernels are built for
// the few tokens of a decoding step; a batch is a sequence of such steps).  Nothing is launched if the first slice,
// which is the largest, is refused.
slim_status dequant_matmul_tokens(slim_ctx* ctx, const char* fn, const uint32_t* packed, int64_t ldp,
                                  const uint32_t* gbits, const int32_t* row_off, const double* scale,
                                  const double* zero, int n, int m, int beta, int bit_base, const void* X,
                                  slim_dtype x_dtype, int64_t t_x, int64_t ldx, float* Y, int64_t ldy, float* fixed,
                                  size_t fixed_floats) {
  SLIM_REQUIRE(ctx, t_x >= 1, "%s: t_x must be at least 1 (got %lld)", fn, (long long)t_x);
  for (int64_t t0 = 0; t0 < t_x; t0 += DQ_MAX_T) {
    const int tc = (int)std::min<int64_t>(DQ_MAX_T, t_x - t0);
    const void* xs = X ? static_cast<const void*>(static_cast<const uint16_t*>(X) + t0 * ldx) : nullptr;
    float* ys = Y ? Y + t0 * ldy : nullptr;
    const slim_status st = dequant_matmul_run(ctx, fn, packed, ldp, gbits, row_off, scale, zero, n, m, beta, bit_base,
                                              xs, x_dtype, tc, ldx, ys, ldy, fixed, fixed_floats);
    if (st != SLIM_OK) return st;
  }
  return SLIM_OK;
}

}  // namespace

size_t slim_ws_need_dequant(int n, int m, int beta, int t_x, int ncu) {
  t_x = std::min(t_x, DQ_MAX_T);
  size_t need = 0;
  for (int mfma = 0; mfma < 2; ++mfma) {       // whichever kernel the activations' type and alignment select
    int gper = 0;
    const int splits = dq_splits(n, m, beta, t_x, std::max(1, ncu), mfma != 0, gper);
    if (splits > 1) need = std::max(need, slim_ws_round(sizeof(float) * (size_t)splits * t_x * n));
  }
  return need;
}

// Device address of this GPU's copy of the fixed buffer: asked for once per device, with that device current
// (slim_create calls this on the context's device), and kept for the life of the process.
slim_status slim_dq_scratch_resolve(slim_ctx* ctx) {
  if (ctx->device < 0 || ctx->device >= DQ_MAX_DEVICES)
    return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "device ordinal %d is beyond the %d this library keeps buffers for",
                     ctx->device, DQ_MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[ctx->device]) {
    int cur = -1;
    SLIM_HIP_TRY(ctx, hipGetDevice(&cur));
    if (cur != ctx->device) return slim_fail(ctx, SLIM_ERR_INVALID_ARG, "the context's device is not the current one");
    float* ptr = nullptr;
    SLIM_HIP_TRY(ctx, hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
    if (!ptr) return slim_fail(ctx, SLIM_ERR_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[ctx->device] = ptr;
  }
  ctx->dq_scratch = g_scratch_ptr[ctx->device];
  return SLIM_OK;
}

extern "C" slim_status slim_dequant_matmul(slim_ctx* ctx, const uint32_t* packed, int64_t ldp, const uint32_t* gbits,
                                           const int32_t* row_off, const double* scale, const double* zero, int n,
                                           int m, int beta, int bit_base, const void* X, slim_dtype x_dtype, int t_x,
                                           int64_t ldx, float* Y, int64_t ldy) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  return dequant_matmul_tokens(ctx, "slim_dequant_matmul", packed, ldp, gbits, row_off, scale, zero, n, m, beta,
                               bit_base, X, x_dtype, t_x, ldx, Y, ldy, nullptr, 0);
}

extern "C" slim_status slim_dequant_matmul_noalloc(slim_ctx* ctx, const uint32_t* packed, int64_t ldp,
                                                 const uint32_t* gbits, const int32_t* row_off, const double* scale,
                                                 const double* zero, int n, int m, int beta, int bit_base,
                                                 const void* X, slim_dtype x_dtype, int t_x, int64_t ldx, float* Y,
                                                 int64_t ldy) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  if (!ctx->dq_scratch) return slim_fail(ctx, SLIM_ERR_HIP, "slim_dequant_matmul_noalloc: the fixed buffer was not resolved");
  // per-kernel event timing creates events on demand, which allocates: it is off for the length of this call
  const bool prof = ctx->prof;
  ctx->prof = false;
  const slim_status st = dequant_matmul_tokens(ctx, "slim_dequant_matmul_noalloc", packed, ldp, gbits, row_off, scale,
                                               zero, n, m, beta, bit_base, X, x_dtype, t_x, ldx, Y, ldy,
                                               ctx->dq_scratch, DQ_SCRATCH_FLOATS);
  ctx->prof = prof;
  return st;
}

// The same layer with the zero points in their packed form (App. B.2: weights AND zeros are stored as packed integers
// and the kernel dequantises both): the zero points are unpacked into the context's workspace (n x k doubles, exact:
// stored value / 2) and the product runs as above, so the result is bit for bit that of slim_dequant_matmul on the
// unpacked zero points.
extern "C" slim_status slim_dequant_matmul_zp(slim_ctx* ctx, const uint32_t* packed, int64_t ldp, const uint32_t* gbits,
                                              const int32_t* row_off, const double* scale, const uint32_t* zpacked,
                                              int64_t ldzp, int zbits, int n, int m, int beta, int bit_base,
                                              const void* X, slim_dtype x_dtype, int t_x, int64_t ldx, float* Y,
                                              int64_t ldy) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  SLIM_REQUIRE(ctx, zpacked != nullptr, "slim_dequant_matmul_zp: null pointer");
  SLIM_REQUIRE(ctx, n > 0 && m > 0 && beta > 0 && m % beta == 0, "slim_dequant_matmul_zp: need n, m > 0 and beta | m");
  SLIM_REQUIRE(ctx, t_x >= 1, "slim_dequant_matmul_zp: t_x must be at least 1");
  const int k = m / beta;
  const size_t need_dq = slim_ws_need_dequant(n, m, beta, t_x, std::max(1, ctx->num_cus));
  const size_t need_z = slim_ws_round(sizeof(double) * (size_t)n * k);
  slim_status st = slim_ws_reserve(ctx, need_dq + need_z);
  if (st != SLIM_OK) return st;
  // the zero points live behind the partial sums, which the product below takes from the start of the workspace
  double* zero = reinterpret_cast<double*>(ctx->ws + need_dq);
  st = slim_unpack_zeros(ctx, zpacked, ldzp, n, k, zbits, zero, k);
  if (st != SLIM_OK) return st;
  return dequant_matmul_tokens(ctx, "slim_dequant_matmul_zp", packed, ldp, gbits, row_off, scale, zero, n, m, beta,
                               bit_base, X, x_dtype, t_x, ldx, Y, ldy, nullptr, 0);
}
