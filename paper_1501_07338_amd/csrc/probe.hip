// Measurement aid: the matrix-core rate this chip sustains with no memory traffic at all, to put beside the
// data-sheet peak when a kernel's matrix-core fraction is reported (the clock under sustained MFMA load is
// below the nominal 2.4 GHz).  Every wave issues independent MFMAs back to back on register operands.
#include "common.h"

namespace vcnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr int kThreads = 256;
static constexpr int kChains = 4;  // independent accumulators per wave

template <bool BF16>
__global__ __launch_bounds__(kThreads) void mfma_probe_kernel(float* __restrict__ sink, int iters) {
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[c][q] = 0.f;
  // operands with varied mantissas (power depends on the data; all-zero operands would flatter the clock)
  const float fa = 1.0f + 0.001f * (float)(threadIdx.x % 61), fb = 0.5f + 0.002f * (float)(threadIdx.x % 53);
  if (BF16) {
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = (__bf16)(fa + 0.01f * e), b[e] = (__bf16)(fb - 0.01f * e);
    for (int i = 0; i < iters; ++i)
#pragma unroll
      for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  } else {
    for (int i = 0; i < iters; ++i)
#pragma unroll
      for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa, fb, acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int q = 0; q < 16; ++q) s += acc[c][q];
  sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

vcnn_status launch_mfma_probe(int dtype, int blocks, int iters, float* sink, hipStream_t st) {
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, st, sink, iters);
  else
    hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, st, sink, iters);
  return check_launch("mfma_probe");
}

}  // namespace vcnn
