// Tile machinery shared by the matrix-core kernels (fp32 in, fp32 accumulate, v_mfma_f32_32x32x2_f32).
//
// A block computes a BM x BN tile of C = A * B from BK-deep slabs staged in LDS.  Each wave owns a
// WM x WN sub-tile held as (WM/32) x (WN/32) accumulators of 16 registers.
//
// LDS layout of one operand slab depends on which of its axes is contiguous in memory:
//   KC  (contiguous along the contraction axis k):  [rows][BK + 4]   - filled with 16-byte stores,
//        read back with one 16-byte load per lane that feeds four consecutive MFMA steps;
//   !KC (contiguous along its free axis):           [BK][rows + 8]   - filled with 16-byte stores,
//        read back with one 4-byte load per lane and step.
// Within a group of 8 k-values, MFMA step i (0..3) contracts k = 8t+i on lanes 0-31 and k = 8t+4+i on
// lanes 32-63; both operands use the same permutation, and a sum does not care about the order.
#pragma once
#include <hip/hip_runtime.h>

namespace vcnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int ROWS, int BK, bool KC>
struct LdsTile {
  static constexpr int PITCH = KC ? BK + 4 : ROWS + 8;
  static constexpr int SIZE = KC ? ROWS * PITCH : BK * PITCH;  // floats
  __device__ static __forceinline__ int at(int row, int k) { return KC ? row * PITCH + k : k * PITCH + row; }
};

// Four MFMA steps' worth of one operand fragment for the 32 rows starting at row0.
template <int ROWS, int BK, bool KC>
__device__ __forceinline__ float4 load_frag(const float* tile, int row0, int t, int lane) {
  using L = LdsTile<ROWS, BK, KC>;
  const int l32 = lane & 31, half = lane >> 5;
  if (KC) {
    return *reinterpret_cast<const float4*>(tile + (row0 + l32) * L::PITCH + 8 * t + 4 * half);
  } else {
    const float* p = tile + (8 * t + 4 * half) * L::PITCH + row0 + l32;
    return make_float4(p[0], p[L::PITCH], p[2 * L::PITCH], p[3 * L::PITCH]);
  }
}

template <int BM, int BN, int BK, int TM, int TN, bool A_KC, bool B_KC>
__device__ __forceinline__ void mma_slab(const float* As, const float* Bs, int wm0, int wn0, int lane,
                                         f32x16 (&acc)[TM][TN]) {
#pragma unroll
  for (int t = 0; t < BK / 8; ++t) {
    float4 a[TM], b[TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) a[mi] = load_frag<BM, BK, A_KC>(As, wm0 + mi * 32, t, lane);
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) b[ni] = load_frag<BN, BK, B_KC>(Bs, wn0 + ni * 32, t, lane);
    // Step-major order: consecutive MFMAs write different accumulators, so none waits on its predecessor.
    const float* af = reinterpret_cast<const float*>(a);
    const float* bf = reinterpret_cast<const float*>(b);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi * 4 + i], bf[ni * 4 + i], acc[mi][ni], 0, 0, 0);
  }
}

// Accumulator layout of the 32x32 result: register q of lane l holds row 8*(q/4) + 4*(l/32) + q%4, column l%32.
__device__ __forceinline__ int acc_row(int q, int lane) { return 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3); }

template <int TM, int TN>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[TM][TN]) {
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;
}

// Global -> register -> LDS staging of one operand slab.  The owning kernel fills v[] (from clamped,
// always-valid addresses) and ok[]; store() writes the slab, zeroing the slots that are not ok.
//   KC  operand: slot = (row, 4 k-values if VEC else 1)
//   !KC operand: slot = (k, 4 rows if VEC else 1)
template <int ROWS, int BK, int THREADS, bool KC, bool VEC>
struct Stager {
  static constexpr int W = VEC ? 4 : 1;
  static constexpr int PER_LINE = (KC ? BK : ROWS) / W;         // slots along the contiguous axis
  static constexpr int LINES_PER_PASS = THREADS / PER_LINE;     // lines covered by all threads at once
  static constexpr int LINES = KC ? ROWS : BK;
  static constexpr int SLOTS = (LINES + LINES_PER_PASS - 1) / LINES_PER_PASS;
  static_assert(THREADS % PER_LINE == 0, "thread count must tile the contiguous axis");
  using L = LdsTile<ROWS, BK, KC>;

  int c;          // position along the contiguous axis (in elements)
  int line0;      // first line (row for KC, k for !KC) of this thread
  float v[SLOTS][W];
  bool ok[SLOTS];  // false: the slot lies outside the matrix and is stored as zeros

  __device__ __forceinline__ void init(int tid) {
    c = (tid % PER_LINE) * W;
    line0 = tid / PER_LINE;
  }
  __device__ __forceinline__ int line(int e) const { return line0 + e * LINES_PER_PASS; }
  // row / k (within the slab) that slot e, element u refers to
  __device__ __forceinline__ int row_of(int e, int u) const { return KC ? line(e) : c + u; }
  __device__ __forceinline__ int k_of(int e, int u) const { return KC ? c + u : line(e); }

  __device__ __forceinline__ void store(float* tile) const {
#pragma unroll
    for (int e = 0; e < SLOTS; ++e) {
      if (SLOTS * LINES_PER_PASS > LINES && line(e) >= LINES) break;
      float* dst = tile + (KC ? line(e) * L::PITCH + c : line(e) * L::PITCH + c);
      if (VEC) {
        *reinterpret_cast<float4*>(dst) = ok[e] ? make_float4(v[e][0], v[e][1], v[e][2], v[e][3])
                                                : make_float4(0.f, 0.f, 0.f, 0.f);
      } else {
        dst[0] = ok[e] ? v[e][0] : 0.f;
      }
    }
  }
};

}  // namespace vcnn
