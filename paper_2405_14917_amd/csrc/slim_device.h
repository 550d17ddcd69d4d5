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

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v += shfl_xor_f64(v, s);
  return v;
}
__device__ __forceinline__ double wave_min(double v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v = fmin(v, shfl_xor_f64(v, s));
  return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v = fmax(v, shfl_xor_f64(v, s));
  return v;
}
__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, WAVE);
  return v;
}

// value of `v` held by lane `src` (src must be wavefront-uniform)
__device__ __forceinline__ double read_lane_f64(double v, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}

}  // namespace slimdev
