// Internal declarations shared by the translation units of libslim (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cstdarg>
#include <new>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "slim.h"

struct slim_prof_entry {
  std::string name;
  double total_ms = 0.0;
  int launches = 0;
};

struct slim_prof_pending {
  const char* name;
  hipEvent_t start, stop;
};

constexpr int SLIM_NUM_EVENTS = 16;

// What slim_sba_prepare left in the workspace: valid until the next call that uses the workspace.
struct slim_sba_prepared {
  bool valid = false;
  const void* W = nullptr;
  const void* X_s = nullptr;
  const char* ws = nullptr;       // workspace base the results live in
  int w_dtype = 0, x_dtype = 0, n = 0, m = 0, beta = 0, N = 0, objective = 0, q1_mode = 0;
  int64_t ldw = 0, t_s = 0, ldxs = 0;
};

struct slim_ctx {
  hipStream_t stream = nullptr;
  int device = 0;
  int num_cus = 0;                // compute units of the device
  char err[512] = {0};
  // grow-only device workspace with a bump pointer that every entry point resets
  char* ws = nullptr;
  size_t ws_bytes = 0;
  size_t ws_off = 0;
  bool ws_external = false;       // the workspace is the caller's (given to slim_create): never grown, never freed
  // small fixed buffers
  double* tau_default = nullptr;  // device, SLIM_DEFAULT_NCAND doubles
  int ncand_default = 0;
  int* dflags = nullptr;          // device, 64 ints (pivot failures, counters)
  char* hpin = nullptr;           // pinned host staging, SLIM_HPIN_BYTES
  // side streams (default priority) and events for work that overlaps with the main stream inside one call
  hipStream_t side = nullptr, side2 = nullptr, side3 = nullptr;
  bool on_side = false;           // `stream` temporarily names a side stream (profiling entries say so)
  hipEvent_t ev[SLIM_NUM_EVENTS] = {};
  // When set (and profiling is off), the next SLIM_LAUNCH signals this event through the kernel's own completion
  // signal instead of a separate record behind it (one packet less between dependent small kernels); the launch
  // clears it.  slim_attach_flush() records it the ordinary way if no launch took it.
  hipEvent_t attach_event = nullptr;
  bool staging_copy_pending = false;   // a host-to-device copy out of hpin that no one has waited for yet (ev[13])
  slim_sba_prepared sba_prep;
  float* dq_scratch = nullptr;    // this device's copy of the fixed partial-sum buffer of slim_dequant_matmul_noalloc
  // profiling
  bool prof = false;
  std::vector<slim_prof_pending> pending;
  std::vector<hipEvent_t> free_events;
  std::vector<slim_prof_entry> entries;
};

constexpr int SLIM_HPIN_BYTES = 1 << 20;
constexpr int SLIM_MAX_CAND = 1024;

slim_status slim_fail(slim_ctx* ctx, slim_status code, const char* fmt, ...);

// Workspace: reserve() makes sure at least `bytes` are available and rewinds the bump pointer;
// alloc() hands out 256-byte aligned pieces of it.  reserve() may synchronise and reallocate.
slim_status slim_ws_reserve(slim_ctx* ctx, size_t bytes);
void* slim_ws_alloc(slim_ctx* ctx, size_t bytes);
inline size_t slim_ws_round(size_t bytes) { return (bytes + 255) & ~size_t(255); }

// Bytes of workspace each entry point reserves for a layer of the given shape (host only; the entry points use the
// same functions, so slim_workspace_query, their maximum, is exact).  ncu = compute units of the device.
size_t slim_ws_need_gram(int m, int64_t t_c, int ncu);
size_t slim_ws_need_inverse(int m);
size_t slim_ws_need_salience(int n, int m);
size_t slim_ws_need_sba(int n, int m, int beta, int64_t t_s);
size_t slim_ws_need_sqc(int n);
size_t slim_ws_need_gptq(int n, int m);
size_t slim_ws_need_dequant(int n, int m, int beta, int t_x, int ncu);
size_t slim_ws_need_lwc(int n, int m, int beta, int steps);

// Looks up (once per device) the device address of the fixed buffer of slim_dequant_matmul_noalloc (dequant.hip).
slim_status slim_dq_scratch_resolve(slim_ctx* ctx);

// Creates the side streams and their events on first use.
slim_status slim_ensure_side(slim_ctx* ctx);

// Returns a pointer to a process-lifetime copy of "<step>@<kernel function>", the form of a profiling entry's
// name for launch sites that choose among several kernel functions.
const char* slim_prof_name(const char* step, const char* kernel_function);

// Profiling hooks used by SLIM_LAUNCH.
void slim_prof_begin(slim_ctx* ctx, const char* name);
void slim_prof_end(slim_ctx* ctx);

#define SLIM_HIP_TRY(ctx, expr)                                                              \
  do {                                                                                       \
    hipError_t e__ = (expr);                                                                 \
    if (e__ != hipSuccess)                                                                   \
      return slim_fail((ctx), SLIM_ERR_HIP, "%s failed: %s (%s:%d)", #expr,                 \
                       hipGetErrorString(e__), __FILE__, __LINE__);                          \
  } while (0)

// Launches `kernel<<<grid, block, shmem, ctx->stream>>>(args...)`, bracketed by profiling events
// when enabled, and turns a launch error into SLIM_ERR_HIP.
#define SLIM_LAUNCH(ctx, name, kernel, grid, block, shmem, ...)                              \
  do {                                                                                       \
    if ((ctx)->prof) slim_prof_begin((ctx), (name));                                         \
    if ((ctx)->attach_event && !(ctx)->prof) {                                               \
      hipExtLaunchKernelGGL(kernel, (grid), (block), (shmem), (ctx)->stream, nullptr,        \
                            (ctx)->attach_event, 0, __VA_ARGS__);                            \
      (ctx)->attach_event = nullptr;                                                         \
    } else {                                                                                 \
      hipLaunchKernelGGL(kernel, (grid), (block), (shmem), (ctx)->stream, __VA_ARGS__);      \
    }                                                                                        \
    if ((ctx)->prof) slim_prof_end((ctx));                                                   \
    hipError_t e__ = hipGetLastError();                                                      \
    if (e__ != hipSuccess)                                                                   \
      return slim_fail((ctx), SLIM_ERR_HIP, "launch of %s failed: %s", (name),              \
                       hipGetErrorString(e__));                                              \
  } while (0)

#define SLIM_REQUIRE(ctx, cond, ...)                                                         \
  do {                                                                                       \
    if (!(cond)) return slim_fail((ctx), SLIM_ERR_INVALID_ARG, __VA_ARGS__);                 \
  } while (0)

// Records an event that was offered to a launch which did not happen (or happened under profiling).
inline hipError_t slim_attach_flush(slim_ctx* ctx) {
  if (!ctx->attach_event) return hipSuccess;
  hipEvent_t e = ctx->attach_event;
  ctx->attach_event = nullptr;
  return hipEventRecord(e, ctx->stream);
}

inline bool slim_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int slim_cdiv(int64_t a, int64_t b) { return static_cast<int>((a + b - 1) / b); }

// ---- fp64 matrix-core GEMM (dgemm.hip) --------------------------------------------------
// C = alpha * A * op(B) + beta * C  for row-major operands.
//   A: M x K (lda).  trans_b = 0: B is K x N (ldb);  trans_b = 1: B is N x K (ldb).
//   C: M x N (ldc); C2 (optional, ldc2) receives a copy of the result.
//   flags: SLIM_GEMM_UPPER_ONLY skips output tiles that lie entirely below the diagonal (M == N).
//          SLIM_GEMM_A_UPPER / SLIM_GEMM_B_UPPER declare A (M x K, square) / op(B) (K x N, square) upper
//          triangular with zeros below the diagonal so that the K range can be cut.
//          SLIM_GEMM_ONE_PER_CU runs the product as a persistent kernel on all but a few CUs, one workgroup per
//          CU, with an LDS request that lets nothing else share those CUs: for bulk work on a side stream next to
//          a latency-critical chain of small kernels on other streams, which then finds the remaining CUs free.
//          SLIM_GEMM_CHAIN marks a small product on a latency-critical chain that runs beside bulk products of other
//          streams: 64 x 32 tiles, whose 24 KiB of LDS and 80 registers fit on a CU beside two workgroups of the
//          128 x 128 form (LDS is handed out in pieces of 1280 bytes: two times 52 of the 128 pieces are taken, and
//          the 32 KiB of a 64 x 64 tile need 26), so that its workgroups start at once instead of waiting for a
//          bulk tile to end (panels and windows of the factorisation: a quarter less kernel time inside a pass).
// K and N even, all pointers 16-byte aligned, leading dimensions even.
enum { SLIM_GEMM_UPPER_ONLY = 1, SLIM_GEMM_A_UPPER = 2, SLIM_GEMM_B_UPPER = 4, SLIM_GEMM_ONE_PER_CU = 8, SLIM_GEMM_CHAIN = 16 };
struct slim_gemm_desc {
  const double* A;
  const double* B;
  double* C;
  double* C2;
  int M, N, K;
  int flags;
  int64_t lda, ldb, ldc, ldc2;
  double alpha, beta;
};
slim_status slim_dgemm(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc& d);
// One or two products (host descriptors) beside a latency-critical chain on other streams: persistent workgroups
// on all but a few CUs, as with SLIM_GEMM_ONE_PER_CU, in one launch.
// `cus`: the CUs the launch may occupy when every product is edge-free (M % 256 == 0, N % 128 == 0, K % 16 == 0,
// no flags): it then works on 256 x 128 tiles, one workgroup per CU.
slim_status slim_dgemm_reserved(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc* descs, int count,
                                int cus);
// Batched form: `descs` is a device array of `count` descriptors; max_M / max_N bound the grid.
slim_status slim_dgemm_batched(slim_ctx* ctx, const char* name, int trans_b, const slim_gemm_desc* descs_dev,
                               int count, int max_M, int max_N);

// ---- small utilities (util.hip) -----------------------------------------------------------
// dst (fp64, rows x cols, ldd) = exact widening of src (F16 / BF16 / F32 / F64, lds); cols % 4 == 0.
slim_status slim_widen_f64(slim_ctx* ctx, const char* name, const void* src, slim_dtype dt, int rows, int cols,
                           int64_t lds, double* dst, int64_t ldd);
slim_status slim_zero_f64(slim_ctx* ctx, const char* name, double* p, int64_t n);
// *out = sum of v[0..n) in a fixed order (single workgroup)
slim_status slim_sum_f64(slim_ctx* ctx, const char* name, const double* v, int n, double* out);
