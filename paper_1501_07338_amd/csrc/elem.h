// Element types of tensors in global memory.  Arithmetic is always done on float values; the
// bfloat16 variant stores x, w, y, dy, dx as 16-bit values (upper half of the float bit pattern,
// round-to-nearest-even on store) and converts when loading and storing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/vcnn.h"

namespace vcnn {

struct bf16 {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const bf16* p) { return bf16_bits_to_f32(p->bits); }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(bf16* p, float v) { p->bits = f32_to_bf16_bits(v); }

// Four consecutive elements; p must be aligned to the size of the group (16 bytes / 8 bytes).
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 ld4(const bf16* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xffff0000u));
}
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void st4(bf16* p, float4 v) {
  uint2 u;
  u.x = (uint32_t)f32_to_bf16_bits(v.x) | ((uint32_t)f32_to_bf16_bits(v.y) << 16);
  u.y = (uint32_t)f32_to_bf16_bits(v.z) | ((uint32_t)f32_to_bf16_bits(v.w) << 16);
  *reinterpret_cast<uint2*>(p) = u;
}

// Four consecutive floats from an address that is only 4-byte aligned: one 16-byte load (the target's unaligned
// access mode serves wide loads at any dword boundary; the compiler emits global_load_dwordx4 for this type).
struct __attribute__((aligned(4))) float4_dword_aligned {
  float x, y, z, w;
};
__device__ __forceinline__ float4 ld4_dword_aligned(const float* p) {
  const float4_dword_aligned t = *reinterpret_cast<const float4_dword_aligned*>(p);
  return make_float4(t.x, t.y, t.z, t.w);
}

// Gradient g passed back through the activation `act` (VCNN_ACT_*) whose forward OUTPUT was y: the factor
// sigma'(.) of the delta recursion, written in terms of y (ReLU: y > 0; tanh: 1 - y^2; sigmoid: y (1 - y)).
__device__ __forceinline__ float act_grad(int act, float y, float g) {
  if (act == VCNN_ACT_RELU) return y > 0.f ? g : 0.f;
  if (act == VCNN_ACT_TANH) return g * (1.f - y * y);
  if (act == VCNN_ACT_SIGMOID) return g * y * (1.f - y);
  return g;
}

// Alignment (in bytes) a pointer needs for ld4 / st4 of its element type.
template <typename T>
__host__ __device__ constexpr unsigned group_bytes() { return 4 * sizeof(T); }
template <typename T>
inline bool group_aligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & (group_bytes<T>() - 1)) == 0; }

}  // namespace vcnn
