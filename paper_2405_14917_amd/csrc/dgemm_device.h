// Device-side pieces of the fp64 matrix-core GEMM that more than one source file builds kernels from.
#ifndef SLIM_DGEMM_DEVICE_H
#define SLIM_DGEMM_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "slim_internal.h"

namespace slimgemm {

typedef double double4v __attribute__((ext_vector_type(4)));
typedef double double2v __attribute__((ext_vector_type(2)));

constexpr int BK = 16, NTHREADS = 256;

// K loop of an interior tile.  A wavefront's 4 * MI * NJ MFMAs of a slab take 64 cycles each; everything else
// an iteration needs is issued in their shadow, in a fixed order: the slab fetched during the previous iteration
// goes from registers to the other LDS stage behind the first MFMAs, the global loads of the slab after it
// follow behind the next ones, and the LDS reads of each k-step of 4 are issued one step ahead.  No clamps and
// no selects: the global pointers just advance by a slab (and stop at the last one, which is then fetched and
// stored again without being used).
// NT threads: NT / 64 wavefronts, two along N and the rest along M.
template <int TRANS_B, int BM, int BN, int NT = NTHREADS>
__device__ __forceinline__ void k_loop_fast(const slim_gemm_desc& d, int row0, int col0, int kbeg, int kend,
                                            double* smem, double4v (&acc)[BM / (NT / 128) / 16][BN / 32]) {
  constexpr int WM = NT / 128;                       // wavefronts along M
  constexpr int MI = BM / WM / 16, NJ = BN / 32;
  constexpr int PA = BM * 8 / NT, PB = BN * 8 / NT;  // double2 per thread and slab
  constexpr int STAGE = BK * BM + BK * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l16 = lane & 15, lk = lane >> 4;

  // A (rows x k in memory): thread -> (row, 2 * PA consecutive k); k-major in LDS
  constexpr int TA = 8 / PA;
  const int ra = tid / TA, kha = (tid % TA) * (2 * PA);
  const double* pa = d.A + (int64_t)(row0 + ra) * d.lda + kbeg + kha;
  const int sa = kha * BM + ra;
  // B: as A when given N x K; else (K x N) thread -> (k, 2 * PB consecutive columns)
  constexpr int TB = 8 / PB, TK = NT / 16;           // threads per row (N x K) or per k (K x N)
  const int rb = TRANS_B ? tid / TB : tid / TK, khb = TRANS_B ? (tid % TB) * (2 * PB) : (tid % TK) * (2 * PB);
  const double* pb = TRANS_B ? d.B + (int64_t)(col0 + rb) * d.ldb + kbeg + khb
                             : d.B + (int64_t)(kbeg + rb) * d.ldb + col0 + khb;
  const int64_t stepb = TRANS_B ? (int64_t)BK : (int64_t)BK * d.ldb;
  const int sb = BK * BM + (TRANS_B ? khb * BN + rb : rb * BN + khb);

  double2v fa[PA], fb[PB];   // (vector types: arrays of HIP's double2 structs end up in scratch)
  constexpr int NST = 2 * PA + (TRANS_B ? 2 * PB : PB);   // LDS stores per slab and thread
  constexpr int NLD = PA + PB;                             // global loads per slab and thread
  auto store_piece = [&](double* st, int p) {
    if (p < 2 * PA) {
      st[sa + p * BM] = (p & 1) ? fa[p >> 1].y : fa[p >> 1].x;
    } else if (TRANS_B) {
      const int q = p - 2 * PA;
      st[sb + q * BN] = (q & 1) ? fb[q >> 1].y : fb[q >> 1].x;
    } else {
      const int q = p - 2 * PA;
      *reinterpret_cast<double2v*>(&st[sb + 2 * q]) = fb[q];
    }
  };
  auto load_piece = [&](int p) {
    if (p < PA)
      fa[p] = reinterpret_cast<const double2v*>(pa)[p];
    else
      fb[p - PA] = reinterpret_cast<const double2v*>(pb)[p - PA];
  };

  const int nslabs = (kend - kbeg) / BK;
  // slab 0 to stage 0, slab 1 (or slab 0 again) into the registers
#pragma unroll
  for (int p = 0; p < NLD; ++p) load_piece(p);
#pragma unroll
  for (int p = 0; p < NST; ++p) store_piece(smem, p);
  if (nslabs > 1) {
    pa += BK;
    pb += stepb;
  }
#pragma unroll
  for (int p = 0; p < NLD; ++p) load_piece(p);
  __syncthreads();

  for (int it = 0; it < nslabs; ++it) {
    const double* as = smem + (it & 1) * STAGE + wm * (BM / WM) + l16;
    const double* bs = smem + (it & 1) * STAGE + BK * BM + wn * (BN / 2) + l16;
    double* other = smem + ((it & 1) ^ 1) * STAGE;
    // the registers hold slab it + 1; the loads below fetch slab min(it + 2, nslabs - 1)
    const bool adv = it + 2 < nslabs;
    const double* pa_next = pa + (adv ? BK : 0);
    const double* pb_next = pb + (adv ? stepb : 0);
    double a[2][MI], b[2][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i) a[0][i] = as[lk * BM + i * 16];
#pragma unroll
    for (int j = 0; j < NJ; ++j) b[0][j] = bs[lk * BN + j * 16];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < BK / 4; ++ks) {
      const int c = ks & 1;
      if (ks + 1 < BK / 4) {
#pragma unroll
        for (int i = 0; i < MI; ++i) a[c ^ 1][i] = as[(4 * (ks + 1) + lk) * BM + i * 16];
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[c ^ 1][j] = bs[(4 * (ks + 1) + lk) * BN + j * 16];
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
          const int g = (ks * MI + i) * NJ + j;      // index of this MFMA within the slab
          if (g < NST) {
            store_piece(other, g);
          } else if (g < NST + NLD) {
            if (g == NST) {
              pa = pa_next;
              pb = pb_next;
            }
            load_piece(g - NST);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
    }
    // a tile with fewer MFMAs per slab than pieces to move issues the rest behind them
    constexpr int NMFMA = (BK / 4) * MI * NJ;
#pragma unroll
    for (int g = NMFMA; g < NST + NLD; ++g) {
      if (g < NST) {
        store_piece(other, g);
      } else {
        if (g == NST) {
          pa = pa_next;
          pb = pb_next;
        }
        load_piece(g - NST);
      }
    }
    __syncthreads();
  }
}

}  // namespace slimgemm

#endif
