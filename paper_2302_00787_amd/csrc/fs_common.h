// Shared device-side helpers of the FAVOR# kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fs {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Device view of an fs_tensor.
struct TensorDev {
  const void* ptr;
  int dtype;            // 0 = f32, 1 = bf16
  long long sb, sh, sl; // element strides
};

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float load_elem(const TensorDev& t, long long idx) {
  return t.dtype == 0 ? ((const float*)t.ptr)[idx] : bf16_bits_to_f32(((const uint16_t*)t.ptr)[idx]);
}

__device__ __forceinline__ void store_elem(const TensorDev& t, long long idx, float v) {
  if (t.dtype == 0) ((float*)t.ptr)[idx] = v;
  else ((uint16_t*)t.ptr)[idx] = f32_to_bf16_bits(v);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Which parameter set serves (b, h) when `groups` sets are given (1, H or B*H of them).
__host__ __device__ __forceinline__ int group_of(int groups, int b, int h, int H) {
  return groups == 1 ? 0 : (groups == H ? h : b * H + h);
}

// Order-preserving map float -> uint32 so that atomicMax on the image is a float max. 0 is below every image.
__device__ __forceinline__ uint32_t float_to_ordered(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

}  // namespace fs
