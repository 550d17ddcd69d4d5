// Small device utilities shared by the entry points: exact widening of 16/32-bit matrices to fp64,
// zero fill, and a fixed-order sum.
#include "slim_device.h"
#include "slim_internal.h"

namespace {

using slimdev::load4;

template <typename T>
__global__ __launch_bounds__(256) void widen_rows(const T* __restrict__ src, int64_t lds, int rows, int cols,
                                                  double* __restrict__ dst, int64_t ldd) {
  const int64_t quads_per_row = cols / 4;
  const int64_t total = (int64_t)rows * quads_per_row;
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = q / quads_per_row;
    const int c = (int)(q % quads_per_row) * 4;
    double v[4];
    load4<T>(src + r * lds + c, v);
    double* o = dst + r * ldd + c;
    *reinterpret_cast<double2*>(o) = make_double2(v[0], v[1]);
    *reinterpret_cast<double2*>(o + 2) = make_double2(v[2], v[3]);
  }
}

__global__ __launch_bounds__(256) void zero_doubles(double* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0.0;
}

__global__ __launch_bounds__(256) void sum_fixed(const double* __restrict__ v, int n, double* __restrict__ out) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) s += v[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int st = 128; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = red[0];
}

}  // namespace

slim_status slim_widen_f64(slim_ctx* ctx, const char* name, const void* src, slim_dtype dt, int rows, int cols,
                           int64_t lds, double* dst, int64_t ldd) {
  SLIM_REQUIRE(ctx, cols % 4 == 0 && lds % 4 == 0 && ldd % 2 == 0, "%s: column count and leading dimensions must be multiples of 4", name);
  const int grid = (int)std::min<int64_t>(((int64_t)rows * (cols / 4) + 255) / 256, 65536);
  if (grid == 0) return SLIM_OK;
  switch (dt) {
    case SLIM_F16:
      SLIM_LAUNCH(ctx, name, widen_rows<__half>, dim3(grid), dim3(256), 0, static_cast<const __half*>(src), lds, rows, cols, dst, ldd);
      break;
    case SLIM_BF16:
      SLIM_LAUNCH(ctx, name, widen_rows<__hip_bfloat16>, dim3(grid), dim3(256), 0, static_cast<const __hip_bfloat16*>(src), lds, rows, cols, dst, ldd);
      break;
    case SLIM_F32:
      SLIM_LAUNCH(ctx, name, widen_rows<float>, dim3(grid), dim3(256), 0, static_cast<const float*>(src), lds, rows, cols, dst, ldd);
      break;
    case SLIM_F64:
      SLIM_LAUNCH(ctx, name, widen_rows<double>, dim3(grid), dim3(256), 0, static_cast<const double*>(src), lds, rows, cols, dst, ldd);
      break;
    default:
      return slim_fail(ctx, SLIM_ERR_UNSUPPORTED, "%s: unknown dtype %d", name, (int)dt);
  }
  return SLIM_OK;
}

slim_status slim_zero_f64(slim_ctx* ctx, const char* name, double* p, int64_t n) {
  if (n <= 0) return SLIM_OK;
  const int grid = (int)std::min<int64_t>((n + 255) / 256, 65536);
  SLIM_LAUNCH(ctx, name, zero_doubles, dim3(grid), dim3(256), 0, p, n);
  return SLIM_OK;
}

slim_status slim_sum_f64(slim_ctx* ctx, const char* name, const double* v, int n, double* out) {
  SLIM_LAUNCH(ctx, name, sum_fixed, dim3(1), dim3(256), 0, v, n, out);
  return SLIM_OK;
}
