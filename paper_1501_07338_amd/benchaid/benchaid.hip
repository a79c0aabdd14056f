// Measurement aids for the benchmark; NOT part of the layer library and not linked into it.  Built as a
// shared object of its own (libvcnn_benchaid.so) that only the benchmark loads.
//   benchaid_mfma: the matrix-core rate this chip sustains with no memory traffic at all, to put beside the
//     data-sheet peak when a kernel's matrix-core fraction is reported (the clock under sustained MFMA load
//     is below the nominal 2.4 GHz).  Every wave issues independent MFMAs back to back on register operands.
//   benchaid_copy: a plain streaming copy of a known size, the yardstick the HBM traffic counters of a
//     profiler run are scaled by.
//   benchaid_marker: an empty kernel whose grid size numbers the phase that follows it in a kernel trace.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr int kThreads = 256;
static constexpr int kChains = 4;  // independent accumulators per wave

// Pseudo-random bits (a multiplicative hash): operands whose bits differ from lane to lane and from step to step.
__device__ __forceinline__ uint32_t mix(uint32_t v) {
  v ^= v >> 16, v *= 0x7feb352du, v ^= v >> 15, v *= 0x846ca68bu, v ^= v >> 16;
  return v;
}
// a float in [1, 2) (or its negative) with random mantissa bits
__device__ __forceinline__ float unit_float(uint32_t bits) {
  return __uint_as_float(0x3f800000u | (bits & 0x807fffffu));
}

// The same loop with operands that CHANGE from one instruction to the next (eight register operand pairs with
// random mantissas, taken in turn): the power the matrix cores draw, and with it the clock the chip holds,
// depends on how many operand bits toggle, and a layer's operands do toggle.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void benchaid_mfma_toggle_kernel(float* __restrict__ sink, int iters) {
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[c][q] = 0.f;
  const uint32_t seed = mix(blockIdx.x * kThreads + threadIdx.x + 1u);
  if (BF16) {
    bf16x8 a[8], b[8];
#pragma unroll
    for (int v = 0; v < 8; ++v)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a[v][e] = (__bf16)unit_float(mix(seed + 16u * v + e));
        b[v][e] = (__bf16)(unit_float(mix(seed + 16u * v + e + 8u)) * 0.001f);
      }
    for (int i = 0; i < iters; i += 8)
#pragma unroll
      for (int v = 0; v < 8; ++v)
#pragma unroll
        for (int c = 0; c < kChains; ++c)
          acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(v + c) & 7], b[(v + 3 * c) & 7], acc[c], 0, 0, 0);
  } else {
    float a[8], b[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) a[v] = unit_float(mix(seed + 2u * v)), b[v] = unit_float(mix(seed + 2u * v + 1u)) * 0.001f;
    for (int i = 0; i < iters; i += 8)
#pragma unroll
      for (int v = 0; v < 8; ++v)
#pragma unroll
        for (int c = 0; c < kChains; ++c)
          acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[(v + c) & 7], b[(v + 3 * c) & 7], acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int q = 0; q < 16; ++q) s += acc[c][q];
  sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void benchaid_mfma_kernel(float* __restrict__ sink, int iters) {
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

// The fp32 matrix-core loop of a 128 x 128 tile with its operands read from LDS, as the layer kernels read them: per
// 16 instructions a wave reads two 16-byte A fragments and eight 4-byte B words at lane-dependent addresses, and
// the block meets at a barrier every 64 instructions.  STAGED adds what feeds such a loop from memory: per barrier
// interval every thread fetches four 16-byte words of a global array (a few MB: it stays in the L2) and writes them
// to LDS before the barrier.  Three blocks per compute unit (52 KB of LDS each), like the layer kernels.  The rate
// of this loop, not the data-sheet peak, is what a kernel of that structure can approach.
static constexpr int kLdsFedFloats = 52 * 1024 / 4;
template <bool STAGED>
__global__ __launch_bounds__(kThreads) void benchaid_mfma_lds_kernel(float* __restrict__ sink, int iters,
                                                                       const float4* __restrict__ src, int src_count4) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < kLdsFedFloats; i += kThreads) lds[i] = 1.0f + 0.001f * (float)((i * 2654435761u) >> 20);
  __syncthreads();
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[a][b][q] = 0.f;
  const int abase = (lane & 31) * 36 + (lane >> 5) * 4;   // A fragments: rows of 32 + 4 floats
  const int bbase = 4096 + (lane & 31) + (lane >> 5);     // B words: 32 neighbouring words, the upper half one further
  float* const stage = lds + 8448;                        // 4 x 1152 floats, behind everything the loop reads
  float4 sv[4];
  size_t pos = ((size_t)blockIdx.x * 977 + tid) % (size_t)(src_count4 - 4096);
  for (int it = 0; it < iters; ++it) {
    const int off = (it & 7) * 8;
    if (STAGED && (it & 3) == 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) sv[e] = src[pos + e * kThreads];
    }
    float4 af[2];
    af[0] = *reinterpret_cast<const float4*>(lds + abase + off);
    af[1] = *reinterpret_cast<const float4*>(lds + abase + 1152 + off);
    float bf[2][4];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int i = 0; i < 4; ++i) bf[ni][i] = lds[bbase + ni * 64 + (off + i) * 67];
    const float* afl = reinterpret_cast<const float*>(af);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(afl[mi * 4 + i], bf[ni][i], acc[mi][ni], 0, 0, 0);
    if ((it & 3) == 3) {
      if (STAGED) {
#pragma unroll
        for (int e = 0; e < 4; ++e) *reinterpret_cast<float4*>(stage + (tid >> 3) * 36 + (tid & 7) * 4 + e * 1152) = sv[e];
        pos = (pos + 4 * kThreads) % (size_t)(src_count4 - 4096);
      }
      __syncthreads();
    }
  }
  float s = STAGED ? stage[tid] : 0.f;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int q = 0; q < 16; ++q) s += acc[a][b][q];
  sink[(size_t)blockIdx.x * kThreads + tid] = s;
}

// dst[i] = src[i], 16 bytes per thread, grid-stride
__global__ __launch_bounds__(kThreads) void benchaid_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                                 size_t count4) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < count4; i += (size_t)gridDim.x * kThreads)
    dst[i] = src[i];
}

// does nothing; its grid size is what a kernel trace shows
__global__ void benchaid_marker_kernel() {}

extern "C" {

// A phase marker for kernel traces: an empty kernel of `id` blocks of 64 threads (grid size 64 * id in the trace).
int benchaid_marker(int id, void* stream) {
  if (id <= 0 || id > 65535) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(benchaid_marker_kernel, dim3((unsigned)id), dim3(64), 0, (hipStream_t)stream);
  return (int)hipGetLastError();
}

// Launches `blocks` blocks of 4 waves that each issue iters x 4 independent matrix-core instructions (bf16 == 0:
// v_mfma_f32_32x32x2_f32, else v_mfma_f32_32x32x16_bf16); one float per thread is written to sink (DEVICE,
// blocks*256 floats).  *flop (HOST, nullable) receives the flop count of the launch.  Returns 0 or a hipError_t.
// toggle != 0: the operands change from instruction to instruction (iters must then be a multiple of 8).
int benchaid_mfma(int bf16, int toggle, int blocks, int iters, float* sink, double* flop, void* stream) {
  if (blocks <= 0 || iters <= 0 || !sink || (toggle && iters % 8)) return (int)hipErrorInvalidValue;
  if (flop) *flop = (double)blocks * 4 * iters * kChains * (bf16 ? 32768.0 : 4096.0);
  if (toggle && bf16)
    hipLaunchKernelGGL(benchaid_mfma_toggle_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, sink, iters);
  else if (toggle)
    hipLaunchKernelGGL(benchaid_mfma_toggle_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, sink, iters);
  else if (bf16)
    hipLaunchKernelGGL(benchaid_mfma_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, sink, iters);
  else
    hipLaunchKernelGGL(benchaid_mfma_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, sink, iters);
  return (int)hipGetLastError();
}

// Launches `blocks` blocks of the LDS-fed loop (iters x 16 instructions per wave, iters a multiple of 8).  staged != 0:
// with the fetch of new operand words from src (DEVICE, src_count4 >= 8192 16-byte words, readable) into LDS every 64
// instructions; src may be null otherwise.  sink: DEVICE, blocks*256 floats.  *flop (HOST, nullable) receives the
// flop count.  Returns 0 or a hipError_t.
int benchaid_mfma_lds(int staged, int blocks, int iters, float* sink, const void* src, int src_count4, double* flop,
                      void* stream) {
  if (blocks <= 0 || iters <= 0 || iters % 8 || !sink || (staged && (!src || src_count4 < 8192))) return (int)hipErrorInvalidValue;
  if (flop) *flop = (double)blocks * 4 * iters * 16 * 4096.0;
  const size_t lds = (size_t)kLdsFedFloats * sizeof(float);
  static bool opted = false;
  if (!opted) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(benchaid_mfma_lds_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(benchaid_mfma_lds_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return (int)e;
    opted = true;
  }
  if (staged)
    hipLaunchKernelGGL(benchaid_mfma_lds_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), lds, (hipStream_t)stream, sink,
                       iters, (const float4*)src, src_count4);
  else
    hipLaunchKernelGGL(benchaid_mfma_lds_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), lds, (hipStream_t)stream, sink,
                       iters, (const float4*)nullptr, 8192);
  return (int)hipGetLastError();
}

// Copies `bytes` (a multiple of 16; src and dst DEVICE, 16-byte aligned) with one streaming kernel.
int benchaid_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || (bytes & 15)) return (int)hipErrorInvalidValue;
  const size_t count4 = bytes / 16;
  size_t blocks = (count4 + kThreads - 1) / kThreads;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(benchaid_copy_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                     (const float4*)src, (float4*)dst, count4);
  return (int)hipGetLastError();
}

}  // extern "C"
