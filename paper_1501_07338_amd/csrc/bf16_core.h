// What the bfloat16 matrix-core kernels share: the MFMA wrappers and the direct global -> LDS load.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace vcnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Direct global -> LDS load of 16 bytes per lane: lane i of the wave deposits its bytes at lds_base + 16 i
// (lds_base wave-uniform, held in M0).  Issued through inline assembly so that the compiler's wait-count
// pass does not see it: seeing it, it drains every outstanding load before each later LDS read, and the
// fragment prefetch loses its lead.  The kernels wait for these loads themselves (vmcnt(0) before the barrier
// that publishes a tile); the hidden loads only make the compiler's own vmcnt waits more conservative,
// never too short, because loads complete in order.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // M0 is reserved by the compiler; naming it as clobbered is still right
__device__ __forceinline__ void load_to_lds16(const uint4* src, uint4* lds_base) {
  const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)lds_base);  // low half = LDS offset
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(base), "v"(src) : "memory", "m0");
}
#pragma clang diagnostic pop

// v_mfma_f32_32x32x16_bf16 / v_mfma_f32_16x16x32_bf16: lane l holds A[row l % T][8 k-values of group l / T] and
// B[the same 8 k-values][column l % T] (T = 32 or 16) as one 16-byte word each.
__device__ __forceinline__ f32x16 mfma_bf16(uint4 a, uint4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_bf16(uint4 a, uint4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

}  // namespace vcnn
