// Device-side helpers shared by the kernels of libslim: widening loads and wavefront reductions.
#pragma once

#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

namespace slimdev {

constexpr int WAVE = 64;

// ---- 4 consecutive elements of a 16-bit / 32-bit matrix, widened exactly to fp64 ---------------
template <typename T>
__device__ __forceinline__ void load4(const T* p, double out[4]);

template <>
__device__ __forceinline__ void load4<__half>(const __half* p, double out[4]) {
  const uint2 raw = *reinterpret_cast<const uint2*>(p);
  const __half2 a = *reinterpret_cast<const __half2*>(&raw.x);
  const __half2 b = *reinterpret_cast<const __half2*>(&raw.y);
  out[0] = (double)__low2float(a);
  out[1] = (double)__high2float(a);
  out[2] = (double)__low2float(b);
  out[3] = (double)__high2float(b);
}

template <>
__device__ __forceinline__ void load4<__hip_bfloat16>(const __hip_bfloat16* p, double out[4]) {
  const uint2 raw = *reinterpret_cast<const uint2*>(p);
  // a bfloat16 is the upper half of a float
  out[0] = (double)__uint_as_float(raw.x << 16);
  out[1] = (double)__uint_as_float(raw.x & 0xffff0000u);
  out[2] = (double)__uint_as_float(raw.y << 16);
  out[3] = (double)__uint_as_float(raw.y & 0xffff0000u);
}

template <>
__device__ __forceinline__ void load4<float>(const float* p, double out[4]) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x;
  out[1] = v.y;
  out[2] = v.z;
  out[3] = v.w;
}

template <>
__device__ __forceinline__ void load4<double>(const double* p, double out[4]) {
  const double2 a = *reinterpret_cast<const double2*>(p);
  const double2 b = *reinterpret_cast<const double2*>(p + 2);
  out[0] = a.x;
  out[1] = a.y;
  out[2] = b.x;
  out[3] = b.y;
}

// ---- wavefront (64 lanes) reductions: every lane ends up with the result ------------------------
__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, mask, WAVE);
  hi = __shfl_xor(hi, mask, WAVE);
  return __hiloint2double(hi, lo);
}

// value of `v` held by lane `src` (src must be wavefront-uniform)
__device__ __forceinline__ double read_lane_f64(double v, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}

// Data-parallel-primitive moves inside a 16-lane row: vector instructions, where a shuffle goes through the LDS
// hardware (a kernel that reduces once per 1 KiB it reads is bound by that instead of by memory).
template <int CTRL>
__device__ __forceinline__ int dpp_b32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  return __hiloint2double(dpp_b32<CTRL>(__double2hiint(v)), dpp_b32<CTRL>(__double2loint(v)));
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;

struct OpSum { __device__ static double f(double a, double b) { return a + b; } };
struct OpMin { __device__ static double f(double a, double b) { return fmin(a, b); } };
struct OpMax { __device__ static double f(double a, double b) { return fmax(a, b); } };
// lanes 1, 2 apart, then the mirror images inside 8 and 16 lanes, then the four rows by lane reads: the same
// association in every lane
template <typename OP>
__device__ __forceinline__ double wave_allreduce(double v) {
  v = OP::f(v, dpp_f64<DPP_XOR1>(v));
  v = OP::f(v, dpp_f64<DPP_XOR2>(v));
  v = OP::f(v, dpp_f64<DPP_HALF_MIRROR>(v));
  v = OP::f(v, dpp_f64<DPP_MIRROR>(v));
  const double r0 = read_lane_f64(v, 0), r1 = read_lane_f64(v, 16), r2 = read_lane_f64(v, 32), r3 = read_lane_f64(v, 48);
  return OP::f(OP::f(r0, r1), OP::f(r2, r3));
}
__device__ __forceinline__ double wave_sum(double v) { return wave_allreduce<OpSum>(v); }
__device__ __forceinline__ double wave_min(double v) { return wave_allreduce<OpMin>(v); }
__device__ __forceinline__ double wave_max(double v) { return wave_allreduce<OpMax>(v); }
__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, WAVE);
  return v;
}

}  // namespace slimdev
