// a1  Proxy Hessian (Eq. 3; Alg. 1 line 1):  G += X_c X_c^T  on the fp16 / bf16 matrix cores
// (v_mfma_f32_32x32x16), fp32 accumulation.
//
// X is m x t with tokens contiguous, so both operands of X X^T are K-contiguous and the kernel is an
// "NT" product of X with itself.  Only tile pairs (bi <= bj) of the symmetric result are computed.
//
//  * Workgroup tile 256 x 256, 256 threads = 4 wavefronts in 2 x 2, each owning 128 x 128 as 4 x 4 MFMA
//    tiles of 32 x 32 (256 fp32 accumulators per lane).  Per K step of 16 a wavefront reads 8 operand
//    fragments from LDS for 16 MFMAs, which keeps LDS at about half of its bandwidth.
//  * K advances in slabs of 64 tokens (128 bytes per row = one cache line).  General kernel (partial tiles,
//    ragged token counts): two LDS stages, the next slab fetched into registers while the current one is
//    multiplied, rows padded to 72 halves so that the 16-byte operand reads of consecutive rows fall into
//    different banks.  Fast path (whole tiles, whole slabs; every benchmark shape): slabs go from memory to LDS
//    directly, swizzled, into a ring of five 32 KiB units that keeps two and a half slabs on the chip
//    (gram_kernel_ring).
//  * Split-K: every tile is cut into S token ranges.  Workgroup ids run over the tiles fastest, so the chip works
//    on one or two token ranges at a time and all XCDs stream through the same narrow band of X together; which
//    tiles are on the chip together, and on which XCD, is decode_work's business.
//  * Every workgroup writes its partial 256 x 256 tile to a slot of a scratch buffer; a second kernel adds the
//    slots of a tile to G in a fixed order (deterministic, no floating-point atomics) and mirrors the upper
//    triangle.
//  * Balance: workgroups run one per CU in rounds of as many as the chip has CUs.  When the last round would be
//    at most half full, the tiles in it are split further along K so that it is full of shorter workgroups; S is
//    the power of two for which a model of the rounds and of the reduction is shortest (a 4096-wide Gram matrix
//    has 136 tiles: S = 2, one round of 128 tiles x 2 ranges and a round of 8 tiles cut 32 ways).
#include <algorithm>
#include <utility>
#include <vector>

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
  int n_main;          // workgroups that take a whole split of their tile: ids 0 .. n_main-1 (order: decode_work)
  int tiles_main;      // tiles handled that way; the tiles behind them are split `f` ways more
  int f;               // sub-splits per split of a tail tile
  int64_t subchunk;    // tokens per sub-split (multiple of BK)
  float* P;            // partial tiles: [slot][TM][TM]
  int interleave;      // how the tiles are dealt to the XCDs: 0 runs, 1 interleaved, 2 patches per round (decode_work)
  int super;           // tile order: edge of a supertile in tiles, or, negative, minus the height of a band (decode_tile)
  int id_base;         // id of the launch's first workgroup (the ring kernel may be launched round by round)
  int ncu;             // workgroups per round (compute units of the device)
};

// Which piece of work a workgroup has: tile, token range, and the slot its partial tile goes to.  The slots of one
// tile are contiguous.  Workgroup ids run over the tiles fastest and the token ranges slowest: the workgroups that
// are on the chip at the same time then cover every tile for one or two token ranges, so the chip as a whole reads
// a narrow band of X at a time.  With the token range fastest instead (every XCD on a range of its own, the
// requests of a moment spread over all of X) the kernel ran 4 % (m = 4096) to 10 % (m = 11008) slower, although its
// L2s requested less.  Workgroup id mod 8 is the XCD.  Dealings of the tiles to the XCDs (`interleave`):
//   0  runs         XCD x (ids x, x + 8, ...) is given a run of consecutive tiles of the tile order, a compact set that
//                   shares its row blocks in that XCD's L2;
//   1  interleaved  consecutive ids take consecutive tiles, so that every row block is wanted by all XCDs at about
//                   the same time (what the two-stage kernel before the ring needed: it could not hide the time of a
//                   first fetch from HBM, and a fetch that another XCD has just made is served by the memory-side
//                   cache; kept for reference, not chosen by the host any more);
//   2  patches      for launches that are cut into rounds: round r takes the tiles ncu r .. ncu (r + 1) - 1, XCD x the
//                   x-th run of ncu / 8 of them, so that the XCDs of a round work on neighbouring patches.
struct WorkItem {
  int tile;
  int64_t kbeg, kend;
  int64_t slot;
};
__device__ __forceinline__ WorkItem decode_work(const GramArgs& a, int id) {
  WorkItem w;
  if (id < a.n_main) {
    const int split = id / a.tiles_main;
    const int j = id - split * a.tiles_main;
    // j = c + 8 q: class c owns tiles_main / 8 consecutive tiles (one more for the first tiles_main % 8 classes)
    const int c = j % 8, per = a.tiles_main / 8, rest = a.tiles_main % 8;
    if (a.interleave == 2) {
      // a round of ncu workgroups takes ncu consecutive tiles, XCD c the c-th run of ncu / 8 of them
      const int R = a.ncu, whole = (a.tiles_main / R) * R;
      w.tile = (j < whole) ? (j / R) * R + c * (R / 8) + (j % R) / 8 : j;
    } else {
      w.tile = a.interleave ? j : c * per + min(c, rest) + j / 8;
    }
    w.kbeg = (int64_t)split * a.kchunk;
    w.kend = min(a.t, w.kbeg + a.kchunk);
    w.slot = (int64_t)w.tile * a.S + split;
  } else {
    const int j = id - a.n_main;
    const int split = j % a.S, q = j / a.S;
    const int sub = q % a.f, tt = q / a.f;
    w.tile = a.tiles_main + tt;
    const int64_t k0 = (int64_t)split * a.kchunk;
    w.kbeg = k0 + (int64_t)sub * a.subchunk;
    w.kend = min(a.t, min(k0 + a.kchunk, w.kbeg + a.subchunk));
    w.slot = (int64_t)a.n_main + ((int64_t)tt * a.S + split) * a.f + sub;
  }
  return w;
}

// position t in the upper triangle of a square grid, column by column: (bi <= bj)
__device__ __forceinline__ void decode_triangle(int t, int& bi, int& bj) {
  int j = (int)((sqrtf(8.0f * (float)t + 1.0f) - 1.0f) * 0.5f);
  while ((j + 1) * (j + 2) / 2 <= t) ++j;
  while (j * (j + 1) / 2 > t) --j;
  bj = j;
  bi = t - j * (j + 1) / 2;
}

// Tile index -> tile (bi <= bj) of the upper triangle of an nt x nt grid.  Tiles are numbered supertile by
// supertile (SUPER x SUPER tiles, the supertiles column by column over the triangle): a run of consecutive tile
// indices, which is what one XCD works on at a time, then covers a compact patch of tiles that needs few row
// blocks of X per slab, and most of its operand loads hit in that XCD's L2.
// Band order (SUPER = -H): the triangle in bands of H tile rows, every band column by column from its diagonal to
// the right.  A run of 32 consecutive tiles is then a patch of H rows by 32 / H columns (H + 32 / H row blocks of X),
// and consecutive runs are neighbours in the same band, which share its H row blocks.
__device__ __forceinline__ void decode_tile_band(int t, int nt, int H, int& bi, int& bj) {
  for (int r0 = 0; r0 < nt; r0 += H) {
    const int r1 = min(nt, r0 + H), hb = r1 - r0;
    const int cnt = hb * (nt - r0) - hb * (hb - 1) / 2;      // sum over the band's rows of (nt - row)
    if (t < cnt) {
      const int tri = hb * (hb - 1) / 2;                      // columns r0 .. r1 - 2 hold 1, 2, .., hb - 1 tiles
      if (t < tri) {
        int c, x;
        decode_triangle(t, x, c);                             // position t = c (c + 1) / 2 + x, x <= c
        bj = r0 + c;
        bi = r0 + x;
      } else {
        t -= tri;
        bj = r1 - 1 + t / hb;
        bi = r0 + t % hb;
      }
      return;
    }
    t -= cnt;
  }
  bi = bj = 0;   // not reached for t < nt (nt + 1) / 2
}

__device__ __forceinline__ void decode_tile(int t, int nt, int& bi, int& bj, int SUPER) {
  if (SUPER < 0) {
    decode_tile_band(t, nt, -SUPER, bi, bj);
    return;
  }
  const int ns = (nt + SUPER - 1) / SUPER;
  for (int J = 0; J < ns; ++J) {
    const int w = min(SUPER, nt - J * SUPER);          // columns of tiles in supertile column J
    for (int I = 0; I <= J; ++I) {
      const int cnt = (I < J) ? SUPER * w : w * (w + 1) / 2;
      if (t < cnt) {
        if (I < J) {
          bi = I * SUPER + t % SUPER;
          bj = J * SUPER + t / SUPER;
        } else {
          decode_triangle(t, bi, bj);
          bi += I * SUPER;
          bj += J * SUPER;
        }
        return;
      }
      t -= cnt;
    }
  }
  bi = bj = 0;   // not reached for t < nt (nt + 1) / 2
}

// 8 consecutive 16-bit elements of one row starting at token k, read branch-free from a clamped (valid)
// address; `valid` tells whether they belong to the matrix and the chunk.  Rows are ldx >= t elements apart
// with ldx a multiple of 8, so the 16 bytes never leave the row's storage.
__device__ __forceinline__ uint4 load_chunk(const uint16_t* rowp, int64_t k, int64_t klast8) {
  return *reinterpret_cast<const uint4*>(rowp + min(k, klast8));
}

// component-wise select (a ternary on the whole vector is lowered through scratch memory)
__device__ __forceinline__ uint4 keep_if(bool ok, uint4 v) {
  return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}

// zero the elements at positions >= nvalid (0..8) of a chunk
__device__ __forceinline__ uint4 mask_chunk(uint4 v, int nvalid) {
  auto keep = [&](uint32_t w, int e0) -> uint32_t {
    const uint32_t lo = (e0 < nvalid) ? 0x0000ffffu : 0u;
    const uint32_t hi = (e0 + 1 < nvalid) ? 0xffff0000u : 0u;
    return w & (lo | hi);
  };
  return make_uint4(keep(v.x, 0), keep(v.y, 2), keep(v.z, 4), keep(v.w, 6));
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

struct RowPtrs {
  const uint16_t* a[CHUNKS];
  const uint16_t* b[CHUNKS];
  unsigned va, vb;   // bit c: row of chunk c exists
};

struct Slab {
  uint4 a[CHUNKS], b[CHUNKS];
};

__device__ __forceinline__ void fetch_slab(Slab& s, const RowPtrs& rp, int64_t k, int64_t klast8) {
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    s.a[c] = load_chunk(rp.a[c], k, klast8);
    s.b[c] = load_chunk(rp.b[c], k, klast8);
  }
}

// writes a fetched slab to LDS, zeroing what lies outside the matrix or the token range [.., kend)
template <bool RAGGED>
__device__ __forceinline__ void stash_slab(const Slab& s, const RowPtrs& rp, uint16_t* as, uint16_t* bs, int64_t k,
                                           int64_t kend) {
  const int nvalid = (int)max((int64_t)0, min((int64_t)8, kend - k));
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    uint4 xa = s.a[c], xb = s.b[c];
    if (RAGGED) {
      xa = mask_chunk(xa, ((rp.va >> c) & 1u) ? nvalid : 0);
      xb = mask_chunk(xb, ((rp.vb >> c) & 1u) ? nvalid : 0);
    } else {
      xa = keep_if(((rp.va >> c) & 1u) && nvalid == 8, xa);
      xb = keep_if(((rp.vb >> c) & 1u) && nvalid == 8, xb);
    }
    *reinterpret_cast<uint4*>(as + 32 * c * LDS_STRIDE) = xa;
    *reinterpret_cast<uint4*>(bs + 32 * c * LDS_STRIDE) = xb;
  }
}

struct Frags {
  uint4 a[4], b[4];
};

__device__ __forceinline__ void load_frags(Frags& f, const uint16_t* as, const uint16_t* bs, int kk) {
#pragma unroll
  for (int i = 0; i < 4; ++i) f.a[i] = *reinterpret_cast<const uint4*>(as + i * 32 * LDS_STRIDE + kk);
#pragma unroll
  for (int j = 0; j < 4; ++j) f.b[j] = *reinterpret_cast<const uint4*>(bs + j * 32 * LDS_STRIDE + kk);
}

template <bool BF16>
__device__ __forceinline__ void mfma_block(float16v (&acc)[4][4], const Frags& f) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = mfma<BF16>(f.a[i], f.b[j], acc[i][j]);
}

// One slab (64 tokens = 4 K steps of 16).  The operand fragments of step kk + 1 are read from LDS into a
// second register set while the 16 MFMAs of step kk run, so the matrix pipe does not wait for LDS.  Left
// alone, the compiler sinks every read next to its use and the pipe idles one LDS round trip per four MFMAs.
template <bool BF16>
__device__ __forceinline__ void multiply_slab(float16v (&acc)[4][4], const uint16_t* as, const uint16_t* bs) {
  Frags f0, f1;
  load_frags(f0, as, bs, 0);
  load_frags(f1, as, bs, 16);
  mfma_block<BF16>(acc, f0);
  load_frags(f0, as, bs, 32);
  mfma_block<BF16>(acc, f1);
  load_frags(f1, as, bs, 48);
  mfma_block<BF16>(acc, f0);
  mfma_block<BF16>(acc, f1);
  // requested issue order inside this scheduling region: 16 LDS reads, then 16 MFMAs with the next 8 reads
  // spread between them, and so on (mask 0x100 = LDS read, 0x008 = MFMA)
  __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
#pragma unroll
  for (int r = 0; r < 2; ++r) {
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
  }
  __builtin_amdgcn_sched_group_barrier(0x008, 32, 0);
}

template <bool BF16, bool RAGGED>
__global__ __launch_bounds__(NTHREADS) void gram_kernel(GramArgs a) {
  extern __shared__ __align__(16) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const WorkItem wk = decode_work(a, blockIdx.x);
  int bi, bj;
  decode_tile(wk.tile, (a.m + TM - 1) / TM, bi, bj, a.super);
  const int rowA0 = bi * TM, rowB0 = bj * TM;
  const int64_t kbeg = wk.kbeg, kend = wk.kend;
  const int64_t klast8 = ((a.t - 1) / 8) * 8;   // start of the last (possibly partial) 8-token chunk

  // LDS stage s: A slab at smem + s * STAGE, B slab TM * LDS_STRIDE behind it
  constexpr int STAGE = 2 * TM * LDS_STRIDE;

  float16v acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // thread -> chunk (row r0 + 32 c, 16-byte column ch) of both operand slabs, c = 0 .. CHUNKS-1
  const int r0 = tid >> 3, ch = tid & 7;
  RowPtrs rp;
  rp.va = 0;
  rp.vb = 0;
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    const int ra = rowA0 + r0 + 32 * c, rb = rowB0 + r0 + 32 * c;
    rp.a[c] = a.X + (int64_t)min(ra, a.m - 1) * a.ldx;
    rp.b[c] = a.X + (int64_t)min(rb, a.m - 1) * a.ldx;
    rp.va |= (ra < a.m) ? (1u << c) : 0u;
    rp.vb |= (rb < a.m) ? (1u << c) : 0u;
  }
  // this thread's store position inside an LDS slab, and its operand read positions
  const int st_off = r0 * LDS_STRIDE + ch * 8;
  const int l32 = lane & 31, lh = lane >> 5;
  const int rdA = (wm * 128 + l32) * LDS_STRIDE + lh * 8;
  const int rdB = TM * LDS_STRIDE + (wn * 128 + l32) * LDS_STRIDE + lh * 8;
  const int64_t kch = ch * 8;

  // The slab fetched into registers in iteration s is written to the other LDS stage at the end of the
  // iteration and multiplied in iteration s + 1.  The fetch behind the last slab reads clamped addresses
  // and is stashed as zeros.
  Slab sl;
  fetch_slab(sl, rp, kbeg + kch, klast8);
  stash_slab<RAGGED>(sl, rp, smem + st_off, smem + TM * LDS_STRIDE + st_off, kbeg + kch, kend);
  __syncthreads();
  int cur = 0;
  for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
    fetch_slab(sl, rp, k0 + BK + kch, klast8);
    __builtin_amdgcn_sched_barrier(0);   // keep the fetch ahead of, and the stash behind, the MFMA block
    multiply_slab<BF16>(acc, smem + cur * STAGE + rdA, smem + cur * STAGE + rdB);
    __builtin_amdgcn_sched_barrier(0);
    cur ^= 1;
    stash_slab<RAGGED>(sl, rp, smem + cur * STAGE + st_off, smem + cur * STAGE + TM * LDS_STRIDE + st_off,
                       k0 + BK + kch, kend);
    __syncthreads();
  }

  // Accumulator register v of lane l holds C[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32] of its 32 x 32 tile.
  float* P = a.P + wk.slot * (TM * TM);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = wm * 128 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
      if (rowA0 + rl >= a.m) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int cl = wn * 128 + j * 32 + l32;
        if (rowB0 + cl < a.m) P[rl * TM + cl] = acc[i][j][v];
      }
    }
  }
}

// ---- interior fast path -----------------------------------------------------------------------------
// Every tile is complete (m a multiple of 256) and every split covers whole slabs, so nothing is masked.
//
// A wavefront that is alone on its SIMD pays the full issue time of every instruction that does not fit in the
// shadow of the matrix pipe, and measured on this kernel the global loads and the LDS stores of the operand
// slabs together cost as much again as a third of the MFMA time.  So the slabs go from memory to LDS directly
// (global_load_lds_dwordx4): one instruction per 1 KiB instead of a load plus a store, no registers in between,
// and a whole iteration for the data to arrive (the loads of slab s+1 are issued before the MFMAs of slab s).
//
// A direct load writes the 64 lanes' 16 bytes to consecutive LDS addresses, so rows cannot be padded: a row
// of a slab is exactly 128 bytes, and 8 lanes x 8 rows of a wavefront form one contiguous KiB.  Bank conflicts
// of the operand reads are avoided by a swizzle instead, applied on the global side: position p (16-byte unit)
// of row r holds the tokens of chunk p ^ ((r >> 1) & 7).  Sixteen lanes that read the same chunk of sixteen
// consecutive rows then hit sixteen different groups of four banks.
constexpr int FROW = BK;                                               // halves per LDS row

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// One direct load: the 64 lanes' 16 bytes at gbase + voff (uniform 64-bit base, 32-bit lane offset) go to the
// LDS bytes lds_addr + 16 * lane.  Written as asm so that the compiler neither computes 64-bit lane addresses
// for it nor makes later LDS reads of the other stage wait for it; completion is awaited explicitly (vmcnt).
__device__ __forceinline__ void direct_load(unsigned lds_addr, unsigned voff, const char* gbase) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(gbase)
               : "m0");
#else
  (void)lds_addr, (void)voff, (void)gbase;
#endif
}

// operand fragments of K step s: `ap` / `bp` already point at this lane's row and swizzled chunk
__device__ __forceinline__ void load_frags_full(Frags& f, const uint16_t* ap, const uint16_t* bp) {
#pragma unroll
  for (int i = 0; i < 4; ++i) f.a[i] = *reinterpret_cast<const uint4*>(ap + i * 32 * FROW);
#pragma unroll
  for (int j = 0; j < 4; ++j) f.b[j] = *reinterpret_cast<const uint4*>(bp + j * 32 * FROW);
}

// ---- the operand slabs in a ring of five units ----------------------------------------------------------
// 160 KiB of LDS hold two and a half slabs.  Instead of two stages of (A slab, B slab), five units of one operand
// slab (256 rows x 128 bytes = 32 KiB) are used in turn: slab s has its A rows in unit 2s mod 5 and its B rows in
// unit 2s + 1 mod 5.  While slab s is multiplied, the two units that slab s - 1 has just freed take B of slab s + 1
// and A of slab s + 2, so half of the loads are on their way a whole slab longer than with two stages, and the
// other half can go out in the first quarter of the slab without the second half crowding the address path.
constexpr unsigned UNIT_BYTES = TM * FROW * 2;                         // 32 KiB
constexpr size_t kSmemRing = size_t(5) * UNIT_BYTES;

template <bool BF16, int S>
__device__ __forceinline__ void kstep_ring(float16v (&acc)[4][4], const Frags& cf, Frags& nf, const uint16_t* nap,
                                           const uint16_t* nbp, unsigned ldsB, unsigned ldsA,
                                           const unsigned (&off)[CHUNKS], const char* srcB, const char* srcA) {
  constexpr unsigned CHUNK_BYTES = 32 * FROW * 2;
#pragma unroll
  for (int m = 0; m < 16; ++m) {
    acc[m >> 2][m & 3] = mfma<BF16>(cf.a[m >> 2], cf.b[m & 3], acc[m >> 2][m & 3]);
    __builtin_amdgcn_sched_barrier(0);
    if (S < 3 && (m & 1) == 0) {
      const int q = m >> 1;
      if (q < 4)
        nf.a[q] = *reinterpret_cast<const uint4*>(nap + q * 32 * FROW);
      else
        nf.b[q - 4] = *reinterpret_cast<const uint4*>(nbp + (q - 4) * 32 * FROW);
      __builtin_amdgcn_sched_barrier(0);
    }
    const int gm = 16 * S + m;             // index of this MFMA in the iteration
    // One direct load per four MFMAs over the whole slab: B of the next slab in the first half, A of the slab after
    // it in the second.  Measured against loads crowded into the first half or quarter of the slab (one per MFMA or
    // per two, as two stages force them to be): the even rate is 1 to 3 % faster, and the ring as a whole 3.5 % (m =
    // 11008) to 7 % (m = 4096) faster than two stages.
    if ((gm & 3) == 1) {
      const int c = gm >> 2;
      if (c < CHUNKS)
        direct_load(ldsB + c * CHUNK_BYTES, off[c], srcB);
      else
        direct_load(ldsA + (c - CHUNKS) * CHUNK_BYTES, off[c - CHUNKS], srcA);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(NTHREADS) void gram_kernel_ring(GramArgs a) {
  extern __shared__ __align__(16) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const WorkItem wk = decode_work(a, a.id_base + (int)blockIdx.x);
  int bi, bj;
  decode_tile(wk.tile, (a.m + TM - 1) / TM, bi, bj, a.super);
  const int rowA0 = bi * TM, rowB0 = bj * TM;
  const int64_t kbeg = wk.kbeg, kend = wk.kend;
  constexpr int UNIT = TM * FROW;         // halves per unit
  float16v acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int r0 = tid >> 3, ch = tid & 7;
  const int gch = ch ^ ((r0 >> 1) & 7);
  unsigned off[CHUNKS];
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) off[c] = (unsigned)((int64_t)(r0 + 32 * c) * a.ldx * 2 + gch * 16);
  const char* const baseA = reinterpret_cast<const char*>(a.X + (int64_t)rowA0 * a.ldx + kbeg);
  const char* const baseB = reinterpret_cast<const char*>(a.X + (int64_t)rowB0 * a.ldx + kbeg);
  const int wrow = 8 * wave * FROW;
  const int l32 = lane & 31, lh = lane >> 5;
  const int xm = (l32 >> 1) & 7;
  const int rdA = (wm * 128 + l32) * FROW, rdB = (wn * 128 + l32) * FROW;     // inside a unit
  int pos[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) pos[s] = ((2 * s + lh) ^ xm) * 8;
  const unsigned lds0 = (unsigned)__builtin_amdgcn_readfirstlane(
      (int)((unsigned)(uintptr_t)((__attribute__((address_space(3))) uint16_t*)smem) + (unsigned)wrow * 2));
  constexpr unsigned CHUNK_BYTES = 32 * FROW * 2;
  const int64_t nslab = (kend - kbeg) / BK;
  const int64_t last = (nslab - 1) * (BK * 2);     // byte offset of the last slab: loads behind it re-read it

  // prologue: A and B of slab 0 into units 0 and 1, A of slab 1 into unit 2
  {
    const char* a1 = baseA + min((int64_t)(BK * 2), last);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      direct_load(lds0 + c * CHUNK_BYTES, off[c], baseA);
      direct_load(lds0 + UNIT_BYTES + c * CHUNK_BYTES, off[c], baseB);
      direct_load(lds0 + 2 * UNIT_BYTES + c * CHUNK_BYTES, off[c], a1);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int ua = 0;                                      // unit of A of the current slab; B is the next one
  const bool idle = (bi == bj && wm == 1 && wn == 0);   // this wavefront's quarter of a diagonal tile is never read back
  if (idle) {
    // only fetches its share of the slabs and keeps the barriers
    for (int64_t it = 0; it < nslab; ++it) {
      const int unB = (ua + 3 >= 5) ? ua + 3 - 5 : ua + 3;
      const int unA = (ua + 4 >= 5) ? ua + 4 - 5 : ua + 4;
      const char* srcB = baseB + min((it + 1) * (int64_t)(BK * 2), last);
      const char* srcA = baseA + min((it + 2) * (int64_t)(BK * 2), last);
      const unsigned ldsB = lds0 + (unsigned)unB * UNIT_BYTES, ldsA = lds0 + (unsigned)unA * UNIT_BYTES;
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        direct_load(ldsB + c * CHUNK_BYTES, off[c], srcB);
        __builtin_amdgcn_s_sleep(1);
      }
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        direct_load(ldsA + c * CHUNK_BYTES, off[c], srcA);
        __builtin_amdgcn_s_sleep(2);
      }
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      __syncthreads();
      ua = (ua + 2 >= 5) ? ua + 2 - 5 : ua + 2;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    return;
  }
  for (int64_t it = 0; it < nslab; ++it) {
    const int ub = (ua + 1 >= 5) ? ua + 1 - 5 : ua + 1;
    const int unB = (ua + 3 >= 5) ? ua + 3 - 5 : ua + 3;     // takes B of slab it + 1
    const int unA = (ua + 4 >= 5) ? ua + 4 - 5 : ua + 4;     // takes A of slab it + 2
    const char* srcB = baseB + min((it + 1) * (int64_t)(BK * 2), last);
    const char* srcA = baseA + min((it + 2) * (int64_t)(BK * 2), last);
    const unsigned ldsB = lds0 + (unsigned)unB * UNIT_BYTES, ldsA = lds0 + (unsigned)unA * UNIT_BYTES;
    const uint16_t* as = smem + ua * UNIT + rdA;
    const uint16_t* bs = smem + ub * UNIT + rdB;
    Frags f0, f1;
    load_frags_full(f0, as + pos[0], bs + pos[0]);
    __builtin_amdgcn_sched_barrier(0);
    kstep_ring<BF16, 0>(acc, f0, f1, as + pos[1], bs + pos[1], ldsB, ldsA, off, srcB, srcA);
    kstep_ring<BF16, 1>(acc, f1, f0, as + pos[2], bs + pos[2], ldsB, ldsA, off, srcB, srcA);
    kstep_ring<BF16, 2>(acc, f0, f1, as + pos[3], bs + pos[3], ldsB, ldsA, off, srcB, srcA);
    kstep_ring<BF16, 3>(acc, f1, f0, as, bs, ldsB, ldsA, off, srcB, srcA);
    // loads complete in order: all but the last eight (A of slab it + 2) have landed, i.e. A and B of slab it + 1
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    __syncthreads();
    ua = (ua + 2 >= 5) ? ua + 2 - 5 : ua + 2;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  float* P = a.P + wk.slot * (TM * TM);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = wm * 128 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
#pragma unroll
      for (int j = 0; j < 4; ++j) P[rl * TM + wn * 128 + j * 32 + l32] = acc[i][j][v];
    }
  }
}

// G[i][j] += the sum over the slots of the tile (in slot order) for every (i, j) of an upper tile pair;
// mirrored into the lower triangle.  One workgroup per 64 x 64 block of a tile: 16-byte reads of the slots,
// the block itself added to G row by row, its transpose through LDS, so that both sides are written in whole rows.
constexpr int RB = 64;
__global__ __launch_bounds__(256) void gram_reduce(GramArgs a, float* __restrict__ G, int64_t ldg) {
  __shared__ float T[RB][RB + 1];
  const int tile = blockIdx.x;
  const int si = blockIdx.y / (TM / RB), sj = blockIdx.y % (TM / RB);
  int bi, bj;
  decode_tile(tile, (a.m + TM - 1) / TM, bi, bj, a.super);
  if (bi == bj && si > sj) return;                 // below the diagonal: written as the mirror of the block above it
  const int row0 = bi * TM + si * RB, col0 = bj * TM + sj * RB;
  if (row0 >= a.m || col0 >= a.m) return;
  const bool diag = (bi == bj && si == sj);
  int64_t base;
  int count;
  if (tile < a.tiles_main) {
    base = (int64_t)tile * a.S;
    count = a.S;
  } else {
    base = (int64_t)a.n_main + (int64_t)(tile - a.tiles_main) * a.S * a.f;
    count = a.S * a.f;
  }
  // thread -> rows tr, tr + 16, tr + 32, tr + 48 of the block, columns tc .. tc + 3
  const int tr = threadIdx.x >> 4, tc = (threadIdx.x & 15) * 4;
  const float* __restrict__ P = a.P + base * (TM * TM) + (int64_t)(si * RB + tr) * TM + sj * RB + tc;
  float4 acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int p = 0; p < count; ++p) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(P + (int64_t)p * (TM * TM) + q * 16 * TM);
      acc[q].x += v.x;
      acc[q].y += v.y;
      acc[q].z += v.z;
      acc[q].w += v.w;
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    T[tr + 16 * q][tc + 0] = acc[q].x;
    T[tr + 16 * q][tc + 1] = acc[q].y;
    T[tr + 16 * q][tc + 2] = acc[q].z;
    T[tr + 16 * q][tc + 3] = acc[q].w;
  }
  __syncthreads();
  const bool vec = (ldg % 4 == 0) && !diag;        // m is a multiple of 8, so a group of 4 is inside or outside
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int y = tr + 16 * q;
    // the block: G[row0 + y][col0 + tc ..]
    if (row0 + y < a.m && col0 + tc < a.m) {
      float* g = G + (int64_t)(row0 + y) * ldg + col0 + tc;
      if (vec) {
        float4 o = *reinterpret_cast<float4*>(g);
        o.x += acc[q].x;
        o.y += acc[q].y;
        o.z += acc[q].z;
        o.w += acc[q].w;
        *reinterpret_cast<float4*>(g) = o;
      } else {
        const float e[4] = {acc[q].x, acc[q].y, acc[q].z, acc[q].w};
#pragma unroll
        for (int x = 0; x < 4; ++x)
          if (!diag || tc + x >= y) g[x] += e[x];
      }
    }
    // its mirror: G[col0 + y][row0 + tc ..] gets T[tc ..][y]
    if (col0 + y < a.m && row0 + tc < a.m) {
      float* g = G + (int64_t)(col0 + y) * ldg + row0 + tc;
      if (vec) {
        float4 o = *reinterpret_cast<float4*>(g);
        o.x += T[tc + 0][y];
        o.y += T[tc + 1][y];
        o.z += T[tc + 2][y];
        o.w += T[tc + 3][y];
        *reinterpret_cast<float4*>(g) = o;
      } else {
#pragma unroll
        for (int x = 0; x < 4; ++x)
          if (!diag || y > tc + x) g[x] += T[tc + x][y];
      }
    }
  }
}

// Token ranges per tile: the number S (a power of two) for which a model of the launch is shortest.  A workgroup
// takes 1/S of a tile's time; n = tiles * S workgroups run in rounds of one per CU; the tiles of a last round that
// is at most half full are split f ways more, so that it is full of workgroups 1/f as long (m = 4096: 136 tiles,
// S = 2 gives one round plus 8 tiles cut 32 ways; m = 5120: 210 tiles, S = 4 gives 3 1/3 rounds where S = 1 or 2
// leave a fifth of the chip idle); every slot costs its 256 KB twice (written here, read by the reduction).
// Few ranges are better beyond the smaller reduction: each workgroup's fill and drain is paid once per range.
struct GramPlan {
  int S, tail_tiles, f;
  int64_t kchunk, subchunk;
  int64_t nwg;           // workgroups = slots of partial tiles
  double cost;
};

GramPlan gram_plan(int m, int64_t t_c, int ncu) {
  const int nt = slim_cdiv(m, TM);
  const int tiles = nt * (nt + 1) / 2;
  const int64_t iters = (t_c + BK - 1) / BK;
  auto plan_for = [&](int S_try) {
    GramPlan p;
    int S = (int)std::min<int64_t>(S_try, iters);
    p.kchunk = ((iters + S - 1) / S) * BK;
    S = (int)((t_c + p.kchunk - 1) / p.kchunk);
    p.S = S;
    const int64_t n_items = (int64_t)tiles * S;
    const int64_t nsl = p.kchunk / BK;
    p.tail_tiles = 0;
    p.f = 1;
    const int r = (int)(n_items % ncu);
    if (n_items > ncu && r >= S && 2 * r <= ncu) {
      p.tail_tiles = r / S;
      p.f = (int)std::min<int64_t>(ncu / (p.tail_tiles * S), nsl);
      if (p.f < 2) {
        p.tail_tiles = 0;
        p.f = 1;
      }
    }
    p.subchunk = p.kchunk;
    if (p.tail_tiles > 0) {
      p.subchunk = ((nsl + p.f - 1) / p.f) * BK;
      p.f = (int)((p.kchunk + p.subchunk - 1) / p.subchunk);   // every sub-split non-empty
    }
    const int64_t n_main = (int64_t)(tiles - p.tail_tiles) * S;
    const double rounds = (double)((n_main + ncu - 1) / ncu) + (p.tail_tiles > 0 ? 1.0 / p.f : 0.0);
    p.nwg = n_main + (int64_t)p.tail_tiles * S * p.f;
    const double t_wg = 2.0 * TM * TM * (double)p.kchunk / 4.6e12;            // seconds per workgroup at 4.6 TFLOP/s per CU
    p.cost = rounds * t_wg + (double)p.nwg * TM * TM * sizeof(float) / 4.2e12;  // + the reduction's read of the slots
    return p;
  };
  GramPlan best = plan_for(1);
  for (int S_try = 2; S_try <= 1024 && (int64_t)S_try * 4 <= iters; S_try *= 2) {
    const GramPlan p = plan_for(S_try);
    if (p.cost < best.cost * 0.995) best = p;
  }
  return best;
}

}  // namespace

size_t slim_ws_need_gram(int m, int64_t t_c, int ncu) {
  return slim_ws_round(sizeof(float) * (size_t)gram_plan(m, t_c, ncu).nwg * TM * TM);
}

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
  const GramPlan best = gram_plan(m, t_c, ctx->num_cus > 0 ? ctx->num_cus : 256);
  const int S = best.S, tail_tiles = best.tail_tiles, f = best.f;
  const int64_t kchunk = best.kchunk, subchunk = best.subchunk;

  GramArgs a;
  a.X = static_cast<const uint16_t*>(X);
  a.ldx = ldx;
  a.m = m;
  a.t = t_c;
  a.kchunk = kchunk;
  a.S = S;
  a.tiles_main = tiles - tail_tiles;
  a.n_main = a.tiles_main * S;
  a.f = f;
  a.subchunk = subchunk;
  a.id_base = 0;
  a.ncu = ctx->num_cus > 0 ? ctx->num_cus : 256;
  // Which tiles are on the chip together, and on which XCD (decode_work).  Up to 700 tiles: a run of consecutive
  // tiles of the supertile order per XCD (supertiles of 6 x 6, of 8 x 8 from 192 tiles on; measured with the ring
  // kernel at 262144 tokens against 16 x 16 supertiles dealt round the XCDs: m = 8192 13.9 against 14.8 ms, m = 5120
  // 5.53 against 5.71 ms).  Beyond that the launch is cut into rounds (below), and every round takes 256 consecutive
  // tiles of the band order, 32 per XCD: a patch of 4 x 8 tiles with 12 row blocks of X.  Measured at m = 11008 with
  // the L2 counters: hit rate 0.69 and 79 GB fetched per pass in 24.9 ms, against 0.58, 105 GB and 25.2 ms for 16 x 16
  // supertiles dealt round the XCDs, and 0.67, 83 GB, 25.1 ms for runs of 8 x 8 supertiles.
  a.interleave = a.tiles_main >= 700 ? 2 : 0;
  a.super = a.interleave ? -4 : (a.tiles_main >= 192 ? 8 : 6);
  const int64_t nwg = (int64_t)a.n_main + (int64_t)tail_tiles * S * f;

  const size_t pbytes = sizeof(float) * (size_t)nwg * TM * TM;
  slim_status st = slim_ws_reserve(ctx, slim_ws_need_gram(m, t_c, ctx->num_cus > 0 ? ctx->num_cus : 256));
  if (st != SLIM_OK) return st;
  a.P = static_cast<float*>(slim_ws_alloc(ctx, pbytes));

  const bool ragged = (t_c % 8) != 0;
  // fast path: complete tiles, whole slabs in every split, lane offsets inside 32 bits
  const bool full = (m % TM == 0) && (t_c % BK == 0) && (kchunk * S == t_c) &&
                    ((int64_t)(TM - 1) * ldx * 2 + 128 < (int64_t(1) << 32));
  const void* variants[6] = {reinterpret_cast<const void*>(gram_kernel<false, false>),
                             reinterpret_cast<const void*>(gram_kernel<false, true>),
                             reinterpret_cast<const void*>(gram_kernel<true, false>),
                             reinterpret_cast<const void*>(gram_kernel<true, true>),
                             reinterpret_cast<const void*>(gram_kernel_ring<false>),
                             reinterpret_cast<const void*>(gram_kernel_ring<true>)};
  static bool attr_done = false;
  if (!attr_done) {
    for (const void* fn : variants)
      SLIM_HIP_TRY(ctx, hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)std::max(kSmemBytes, kSmemRing)));
    attr_done = true;
  }
  const dim3 grid((unsigned)nwg), block(NTHREADS);
  // Launches of the fast path.  Workgroups that share row blocks of X find each other's lines in their XCD's L2 only
  // while they are at the same tokens, i.e. while they have started together; a workgroup that starts when another
  // one ends (diagonal tiles end 14 % early) shares nothing.  With many rounds of workgroups the starts drift apart,
  // so a long launch is cut into launches of one round each: the end of a launch is the point where all start
  // together again.  Measured at 262144 tokens: m = 11008 (7.4 rounds) 25.8 against 27.4 ms, m = 12288 32.3 against
  // 34.8 ms, m = 16384 (131072 tokens) 28.5 against 30.3 ms; with three rounds or fewer the ends of the launches cost
  // what the lockstep gains (m = 5120: 5.76 against 5.52 ms), so short launches stay whole.
  const int ncu_l = ctx->num_cus > 0 ? ctx->num_cus : 256;
  std::vector<std::pair<int64_t, int64_t>> rounds;     // (first workgroup id, workgroups)
  if (full && (int64_t)a.n_main >= 5 * (int64_t)ncu_l) {
    int64_t base = 0;
    for (; base + 2 * ncu_l <= nwg; base += ncu_l) rounds.emplace_back(base, (int64_t)ncu_l);
    rounds.emplace_back(base, nwg - base);             // the rest of the last full round with the short tail workgroups
  } else {
    rounds.emplace_back((int64_t)0, nwg);
  }
  if (x_dtype == SLIM_BF16) {
    if (full) {
      for (const auto& r : rounds) {
        a.id_base = (int)r.first;
        SLIM_LAUNCH(ctx, "gram_mfma_bf16@gram_kernel_ring<true>", (gram_kernel_ring<true>), dim3((unsigned)r.second), block,
                    kSmemRing, a);
      }
    } else if (ragged)
      SLIM_LAUNCH(ctx, "gram_mfma_bf16@gram_kernel<true, true>", (gram_kernel<true, true>), grid, block, kSmemBytes, a);
    else
      SLIM_LAUNCH(ctx, "gram_mfma_bf16@gram_kernel<true, false>", (gram_kernel<true, false>), grid, block, kSmemBytes, a);
  } else {
    if (full) {
      for (const auto& r : rounds) {
        a.id_base = (int)r.first;
        SLIM_LAUNCH(ctx, "gram_mfma_f16@gram_kernel_ring<false>", (gram_kernel_ring<false>), dim3((unsigned)r.second), block,
                    kSmemRing, a);
      }
    } else if (ragged)
      SLIM_LAUNCH(ctx, "gram_mfma_f16@gram_kernel<false, true>", (gram_kernel<false, true>), grid, block, kSmemBytes, a);
    else
      SLIM_LAUNCH(ctx, "gram_mfma_f16@gram_kernel<false, false>", (gram_kernel<false, false>), grid, block, kSmemBytes, a);
  }
  SLIM_LAUNCH(ctx, "gram_reduce", gram_reduce, dim3(tiles, (TM / RB) * (TM / RB)), dim3(256), 0, a, G, ldg);
  *n_tokens += t_c;
  return SLIM_OK;
}
