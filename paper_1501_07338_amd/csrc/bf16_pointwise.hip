// Unpadded 1 x 1 layers of the bf16 variant as plain bf16 matrix-core products, straight from the NCHW tensors.
// For such a layer the patch matrix of Eq. 2 is the input itself, so the three passes are three dense products:
//     forward          y[n][m][p]  = sum_c w[m][c] * x[n][c][p]              (+ bias, sigma)
//     input gradient   dx[n][c][p] = sum_m w[m][c] * dy[n][m][p]             (the same kernel on the transposed matrix)
//     kernel gradient  dw[m][c]    = sum_n sum_p dy[n][m][p] * x[n][c][p]
// v_mfma_f32_32x32x16_bf16 wants, in every lane, eight CONSECUTIVE contraction elements of one row / column.  The
// kernel matrix has them (its rows are contraction-contiguous), and so have both operands of the kernel gradient
// (the contraction runs over the pixels).  The activations of the first two products do not: their contraction
// index is the channel, strided by the plane size.  They are transposed on the way into LDS - a thread fetches
// 8 channels x 4 pixels and writes, per pixel, its 8 channels as one 16-byte word - so no re-laid copy of the
// activations is ever written to memory.
//
// Rows of a plane start at any 2-byte boundary (odd pixel counts).  Global loads here are dword-aligned: a group
// that starts on an odd element is fetched from the aligned dword below it, one dword more, and shifted down by
// 16 bits; every dword that is loaded contains at least one element of the tensor.
#include <algorithm>

#include "common.h"
#include "elem.h"

namespace vcnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int kThreads = 256;
static constexpr int kSlabK = 64;          // contraction elements per LDS slab
static constexpr int kPitch = kSlabK + 8;  // bf16 elements per LDS row: 16-byte aligned rows, conflict-free 16-byte reads

__device__ __forceinline__ f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ int acc_row16(int q, int lane) { return 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3); }

// The aligned dword at or below element address p, and whether p is its upper half.  (Pointer arithmetic, not a
// round trip through an integer: the result must still be known to point to global memory.)
__device__ __forceinline__ const uint32_t* dword_below(const bf16* p, uint32_t* odd) {
  *odd = (uint32_t)(reinterpret_cast<uintptr_t>(p) >> 1) & 1u;
  return reinterpret_cast<const uint32_t*>(p - *odd);
}
// Work item of workgroup `block` when the `total` items are dealt to the eight XCDs in contiguous eighths (workgroups
// go to the XCDs in turn); negative for the padding workgroups of a grid rounded up to a multiple of eight.
static constexpr int kXcds = 8;
__device__ __forceinline__ int xcd_chunked(int block, int total) {
  const int chunk = (total + kXcds - 1) / kXcds;
  const int item = (block % kXcds) * chunk + block / kXcds;
  return block / kXcds < chunk && item < total ? item : -1;
}
inline int64_t xcd_grid(int64_t total) { return ceil_div(total, kXcds) * kXcds; }

// (hi:lo) >> (16 * odd), low 32 bits
__device__ __forceinline__ uint32_t shift16(uint32_t lo, uint32_t hi, uint32_t odd) {
  return __builtin_amdgcn_alignbit(hi, lo, 16u * odd);
}
// Up to `count` (< the group size) elements from p, one at a time, zeros behind them.
template <int GROUP>
__device__ __forceinline__ void load_some(const bf16* p, int count, uint32_t* out) {
#pragma unroll
  for (int j = 0; j < GROUP / 2; ++j) {
    const uint32_t lo = 2 * j < count ? (uint32_t)p[2 * j].bits : 0u;
    const uint32_t hi = 2 * j + 1 < count ? (uint32_t)p[2 * j + 1].bits : 0u;
    out[j] = lo | (hi << 16);
  }
}

// ---- y[n][i][p] = act(bias[i] + sum_k A[i][k] * X[n][k][p]) ----------------------------------------------------------
struct PointwiseBf16Args {
  const bf16* A;      // [M][K], rows contraction-contiguous and 16-byte aligned (K % 8 == 0)
  const bf16* X;      // [n][K][P]
  const float* bias;  // [M] or null
  bf16* Y;            // [n][M][P]
  int n, M, K, P;
  int tiles_m, tiles_p;
  int relu;
};

// The product for planes of at least one pixel tile and contractions that are whole slabs: nothing in the loop
// depends on the shape.  A tile that would run over the end of the plane starts early instead (it overlaps its
// neighbour and stores only its own pixels), so every group of four pixels is whole; the dword index and the parity
// of a thread's eight rows are the same in every slab (a slab is 64 rows = 32 * P dwords further on).
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void pointwise_bf16_fast_kernel(PointwiseBf16Args a) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  static_assert(BN == 128, "a thread stages 8 channels x 4 pixels: 32 threads cover 128 pixels");
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_SLAB = BM * kPitch;
  constexpr int ROWS_PER_PASS = kThreads / 8;
  constexpr int A_SLOTS = BM / ROWS_PER_PASS;
  extern __shared__ uint4 smem16[];
  bf16* const As = reinterpret_cast<bf16*>(smem16);  // one slab of each operand: the next one waits in registers
  bf16* const Bs = As + A_SLAB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // consecutive workgroups go to different XCDs (each with an L2 of its own): XCD x takes the x-th eighth of the
  // tiles, so that the row tiles of one pixel tile, which read the same activations, share an L2
  const int bid = xcd_chunked(blockIdx.x, a.tiles_m * a.n * a.tiles_p);
  if (bid < 0) return;
  const int tm = bid % a.tiles_m;
  const int tj = bid / a.tiles_m;
  const int n = tj / a.tiles_p;
  const int p_own = (tj - n * a.tiles_p) * BN;  // the tile's own first pixel
  const int p0 = min(p_own, a.P - BN);          // where it starts reading
  const int i0 = tm * BM;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const bf16* const xn = a.X + (int64_t)n * a.K * a.P;
  const uint32_t xpar = (uint32_t)(reinterpret_cast<uintptr_t>(xn) >> 1) & 1u;
  const uint32_t* const xal = reinterpret_cast<const uint32_t*>(xn - xpar);  // dword-aligned

  const int piece = tid & 7, row0 = tid >> 3;
  const int kg = tid >> 5, pg = tid & 31;
  uint32_t aoff[A_SLOTS];
#pragma unroll
  for (int e = 0; e < A_SLOTS; ++e) aoff[e] = (uint32_t)min(i0 + row0 + e * ROWS_PER_PASS, a.M - 1) * a.K + piece * 8;
  uint32_t xd[8], xodd = 0u;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t idx = xpar + (uint32_t)(8 * kg + j) * a.P + p0 + 4 * pg;
    xd[j] = idx >> 1;
    xodd |= (idx & 1u) << j;
  }

  u32x4 areg[A_SLOTS];
  uint32_t xraw[8][3];
  auto fetch = [&](int sl) {
    const bf16* as = a.A + sl * kSlabK;
    const uint32_t* xs = xal + (size_t)sl * (kSlabK / 2) * a.P;
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e) areg[e] = *reinterpret_cast<const u32x4*>(as + aoff[e]);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t odd = (xodd >> j) & 1u;
      xraw[j][0] = xs[xd[j]], xraw[j][1] = xs[xd[j] + 1];
      xraw[j][2] = xs[xd[j] + 1 + odd];  // the dword with the fourth element of a row that starts on an odd one
    }
  };
  auto store = [&]() {
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e)
      *reinterpret_cast<u32x4*>(As + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) = areg[e];
    uint2 xreg[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t odd = (xodd >> j) & 1u;
      xreg[j] = make_uint2(shift16(xraw[j][0], xraw[j][1], odd), shift16(xraw[j][1], xraw[j][2], odd));
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x4 w;
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const uint32_t lo = q < 2 ? xreg[2 * m].x : xreg[2 * m].y;
        const uint32_t hi = q < 2 ? xreg[2 * m + 1].x : xreg[2 * m + 1].y;
        w[m] = (q & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
      }
      *reinterpret_cast<u32x4*>(Bs + (4 * pg + q) * kPitch + kg * 8) = w;
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  // this thread's rows of the bias, requested before the loop
  float bias_r[TM][16];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int q = 0; q < 16; ++q)
      bias_r[mi][q] = a.bias ? a.bias[min(i0 + wm0 + mi * 32 + acc_row16(q, lane), a.M - 1)] : 0.f;

  const int slabs = a.K / kSlabK;
  fetch(0);
  store();
  __syncthreads();
  for (int sl = 0; sl < slabs; ++sl) {
    const bool more = sl + 1 < slabs;
    if (more) fetch(sl + 1);
#pragma unroll
    for (int i = 0; i < kSlabK / 16; ++i) {
      u32x4 af[TM], bfr[TN];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
        af[mi] = *reinterpret_cast<const u32x4*>(As + (wm0 + mi * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
        bfr[ni] = *reinterpret_cast<const u32x4*>(Bs + (wn0 + ni * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(af[mi], bfr[ni], acc[mi][ni]);
    }
    __syncthreads();  // every wave has read the slab
    if (more) store();
    __syncthreads();
  }

  bf16* const yn = a.Y + (int64_t)n * a.M * a.P;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = p0 + wn0 + ni * 32 + l32;
    if (p < p_own) continue;  // the neighbour's pixels
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row16(q, lane);
        if (i < a.M) {
          float v = acc[mi][ni][q] + bias_r[mi][q];
          if (a.relu) v = fmaxf(v, 0.f);
          st(yn + (int64_t)i * a.P + p, v);
        }
      }
  }
}

// Any plane size and any contraction that is a multiple of 8 (small layers).
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void pointwise_bf16_kernel(PointwiseBf16Args a) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  static_assert(BN == 128, "a thread stages 8 channels x 4 pixels: 32 threads cover 128 pixels");
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_SLAB = BM * kPitch, B_SLAB = BN * kPitch;
  constexpr int ROWS_PER_PASS = kThreads / 8;
  constexpr int A_SLOTS = BM / ROWS_PER_PASS;
  extern __shared__ uint4 smem16[];
  bf16* const As0 = reinterpret_cast<bf16*>(smem16);
  bf16* const Bs0 = As0 + 2 * A_SLAB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // consecutive workgroups go to different XCDs (each with an L2 of its own): XCD x takes the x-th eighth of the
  // tiles, so that the row tiles of one pixel tile, which read the same activations, share an L2
  const int bid = xcd_chunked(blockIdx.x, a.tiles_m * a.n * a.tiles_p);
  if (bid < 0) return;
  const int tm = bid % a.tiles_m;
  const int tj = bid / a.tiles_m;
  const int n = tj / a.tiles_p;
  const int p0 = (tj - n * a.tiles_p) * BN;
  const int i0 = tm * BM;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const bf16* const xn = a.X + (int64_t)n * a.K * a.P;

  // A: a thread fetches 16 bytes (8 contraction elements) of A_SLOTS rows
  const int piece = tid & 7, row0 = tid >> 3;
  // X: a thread fetches 4 pixels of 8 channels
  const int kg = tid >> 5, pg = tid & 31;
  const int px = p0 + 4 * pg;
  const int px_count = min(4, a.P - px);  // <= 0: beyond the plane

  // fetch() only issues the loads; whatever uses a loaded value (masks, the 16-bit shift of rows that start on an
  // odd element) waits until store(), after the slab's MFMAs, so that the loads have the whole slab to arrive
  u32x4 areg[A_SLOTS];
  uint32_t aok = 0u;
  uint32_t xraw[8][3];
  uint32_t xodd = 0u;
  auto fetch = [&](int k0) {
    const int k = k0 + piece * 8;
    const bool kin = k < a.K;
    aok = 0u, xodd = 0u;
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e) {
      const int i = i0 + row0 + e * ROWS_PER_PASS;
      areg[e] = *reinterpret_cast<const u32x4*>(a.A + (int64_t)min(i, a.M - 1) * a.K + (kin ? k : 0));
      aok |= (kin && i < a.M ? 1u : 0u) << e;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int kk = k0 + 8 * kg + j;
      xraw[j][0] = xraw[j][1] = xraw[j][2] = 0u;
      if (kk < a.K && px_count > 0) {
        const bf16* src = xn + (int64_t)kk * a.P + px;
        if (px_count == 4) {
          uint32_t odd;
          const uint32_t* q = dword_below(src, &odd);
          xraw[j][0] = q[0], xraw[j][1] = q[1];
          if (odd) xraw[j][2] = q[2];  // elements 3 and 4: needed, and certainly inside the tensor, only then
          xodd |= odd << j;
        } else {
          load_some<4>(src, px_count, xraw[j]);
        }
      }
    }
  };
  auto store = [&](bf16* As, bf16* Bs) {
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e) {
      u32x4 v = areg[e];
      if (!((aok >> e) & 1u)) v = u32x4{0u, 0u, 0u, 0u};
      *reinterpret_cast<u32x4*>(As + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) = v;
    }
    uint2 xreg[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t odd = (xodd >> j) & 1u;
      xreg[j] = make_uint2(shift16(xraw[j][0], xraw[j][1], odd), shift16(xraw[j][1], xraw[j][2], odd));
    }
    // transpose 8 channels x 4 pixels: pixel q's eight channels become one 16-byte word
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x4 w;
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const uint32_t lo = q < 2 ? xreg[2 * m].x : xreg[2 * m].y;
        const uint32_t hi = q < 2 ? xreg[2 * m + 1].x : xreg[2 * m + 1].y;
        w[m] = (q & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
      }
      *reinterpret_cast<u32x4*>(Bs + (4 * pg + q) * kPitch + kg * 8) = w;
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  const int slabs = (a.K + kSlabK - 1) / kSlabK;
  fetch(0);
  store(As0, Bs0);
  __syncthreads();
  for (int sl = 0; sl < slabs; ++sl) {
    const int cur = sl & 1;
    const bool more = sl + 1 < slabs;
    if (more) fetch((sl + 1) * kSlabK);
    const bf16* As = As0 + cur * A_SLAB;
    const bf16* Bs = Bs0 + cur * B_SLAB;
#pragma unroll
    for (int i = 0; i < kSlabK / 16; ++i) {
      u32x4 af[TM], bfr[TN];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
        af[mi] = *reinterpret_cast<const u32x4*>(As + (wm0 + mi * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
        bfr[ni] = *reinterpret_cast<const u32x4*>(Bs + (wn0 + ni * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(af[mi], bfr[ni], acc[mi][ni]);
    }
    if (more) store(As0 + (cur ^ 1) * A_SLAB, Bs0 + (cur ^ 1) * B_SLAB);
    __syncthreads();
  }

  bf16* const yn = a.Y + (int64_t)n * a.M * a.P;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = p0 + wn0 + ni * 32 + l32;
    if (p >= a.P) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row16(q, lane);
        if (i < a.M) {
          float v = acc[mi][ni][q];
          if (a.bias) v += a.bias[i];
          if (a.relu) v = fmaxf(v, 0.f);
          st(yn + (int64_t)i * a.P + p, v);
        }
      }
  }
}

// ---- out[split][i][j] = sum over the split's (sample, pixel) range of U[n][i][p] * V[n][j][p] ------------------------
struct PointwiseFilterBf16Args {
  const bf16* U;  // [n][M][P]   (dy)
  const bf16* V;  // [n][C][P]   (x)
  float* out;     // [splits][M][C]
  int n, M, C, P;
  int tiles_m, tiles, splits;
  int slabs_per_img;    // ceil(P / kSlabK)
  int units_per_split;  // (sample, slab) units per split
};

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void pointwise_filter_bf16_kernel(PointwiseFilterBf16Args a) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_SLAB = BM * kPitch, B_SLAB = BN * kPitch;
  constexpr int ROWS_PER_PASS = kThreads / 8;
  constexpr int A_SLOTS = BM / ROWS_PER_PASS, B_SLOTS = BN / ROWS_PER_PASS;
  extern __shared__ uint4 smem16[];
  bf16* const As0 = reinterpret_cast<bf16*>(smem16);
  bf16* const Bs0 = As0 + 2 * A_SLAB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // XCD x takes the x-th eighth of the (split, tile) pairs: the tiles of one split, which read the same pixels of
  // both operands, share an L2
  const int bid = xcd_chunked(blockIdx.x, a.tiles * a.splits);
  if (bid < 0) return;
  const int tile = bid % a.tiles, split = bid / a.tiles;
  const int i0 = (tile % a.tiles_m) * BM;
  const int j0 = (tile / a.tiles_m) * BN;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int piece = tid & 7, row0 = tid >> 3;
  const int total_units = a.n * a.slabs_per_img;
  const int u0 = split * a.units_per_split;
  const int u1 = min(total_units, u0 + a.units_per_split);

  // fetch() only issues the loads (five raw dwords per group of eight pixels); the 16-bit shift of groups that start
  // on an odd element happens in store(), after the slab's MFMAs
  uint32_t raw[A_SLOTS + B_SLOTS][5];
  uint32_t oddmask = 0u;
  // eight pixels of one row of one sample, zeros beyond the plane or beyond the operand's last row
  auto group = [&](const bf16* base, int rows, int n, int row, int p, uint32_t* r, int slot) {
    r[0] = r[1] = r[2] = r[3] = r[4] = 0u;
    const int count = min(8, a.P - p);
    if (row < rows && count > 0) {
      const bf16* src = base + ((int64_t)n * rows + row) * a.P + p;
      if (count == 8) {
        uint32_t odd;
        const uint32_t* q = dword_below(src, &odd);
        r[0] = q[0], r[1] = q[1], r[2] = q[2], r[3] = q[3];
        if (odd) r[4] = q[4];
        oddmask |= odd << slot;
      } else {
        load_some<8>(src, count, r);
      }
    }
  };
  auto fetch = [&](int u) {
    const int n = u / a.slabs_per_img;
    const int p = (u - n * a.slabs_per_img) * kSlabK + piece * 8;
    oddmask = 0u;
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e) group(a.U, a.M, n, i0 + row0 + e * ROWS_PER_PASS, p, raw[e], e);
#pragma unroll
    for (int e = 0; e < B_SLOTS; ++e) group(a.V, a.C, n, j0 + row0 + e * ROWS_PER_PASS, p, raw[A_SLOTS + e], A_SLOTS + e);
  };
  auto shifted = [&](int slot) -> u32x4 {
    const uint32_t odd = (oddmask >> slot) & 1u;
    const uint32_t* r = raw[slot];
    return u32x4{shift16(r[0], r[1], odd), shift16(r[1], r[2], odd), shift16(r[2], r[3], odd), shift16(r[3], r[4], odd)};
  };
  auto store = [&](bf16* As, bf16* Bs) {
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e)
      *reinterpret_cast<u32x4*>(As + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) = shifted(e);
#pragma unroll
    for (int e = 0; e < B_SLOTS; ++e)
      *reinterpret_cast<u32x4*>(Bs + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) = shifted(A_SLOTS + e);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  if (u0 < u1) {
    fetch(u0);
    store(As0, Bs0);
  }
  __syncthreads();
  for (int u = u0; u < u1; ++u) {
    const int cur = (u - u0) & 1;
    const bool more = u + 1 < u1;
    if (more) fetch(u + 1);
    const bf16* As = As0 + cur * A_SLAB;
    const bf16* Bs = Bs0 + cur * B_SLAB;
#pragma unroll
    for (int i = 0; i < kSlabK / 16; ++i) {
      u32x4 af[TM], bfr[TN];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
        af[mi] = *reinterpret_cast<const u32x4*>(As + (wm0 + mi * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
        bfr[ni] = *reinterpret_cast<const u32x4*>(Bs + (wn0 + ni * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(af[mi], bfr[ni], acc[mi][ni]);
    }
    if (more) store(As0 + (cur ^ 1) * A_SLAB, Bs0 + (cur ^ 1) * B_SLAB);
    __syncthreads();
  }

  float* dst = a.out + (int64_t)split * a.M * a.C;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int j = j0 + wn0 + ni * 32 + l32;
    if (j >= a.C) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row16(q, lane);
        if (i < a.M) dst[(int64_t)i * a.C + j] = acc[mi][ni][q];
      }
  }
}

// The same product for planes of at least one slab (64 pixels).  The last slab of a sample, which would run over the
// end of the plane, covers the plane's LAST 64 pixels instead and masks those the slab before it has already
// contracted, so every group of eight pixels is whole and inside the tensor.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void pointwise_filter_bf16_fast_kernel(PointwiseFilterBf16Args a) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_SLAB = BM * kPitch;
  constexpr int ROWS_PER_PASS = kThreads / 8;
  constexpr int A_SLOTS = BM / ROWS_PER_PASS, B_SLOTS = BN / ROWS_PER_PASS, SLOTS = A_SLOTS + B_SLOTS;
  extern __shared__ uint4 smem16[];
  bf16* const As = reinterpret_cast<bf16*>(smem16);  // one slab of each operand: the next one waits in registers
  bf16* const Bs = As + A_SLAB;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // XCD x takes the x-th eighth of the (split, tile) pairs: the tiles of one split, which read the same pixels of
  // both operands, share an L2
  const int bid = xcd_chunked(blockIdx.x, a.tiles * a.splits);
  if (bid < 0) return;
  const int tile = bid % a.tiles, split = bid / a.tiles;
  const int i0 = (tile % a.tiles_m) * BM;
  const int j0 = (tile / a.tiles_m) * BN;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int piece = tid & 7, row0 = tid >> 3;
  const int total_units = a.n * a.slabs_per_img;
  const int u0 = split * a.units_per_split;
  const int u1 = min(total_units, u0 + a.units_per_split);

  // element offset of a slot's row inside a sample (rows beyond the operand are clamped: their products are not stored)
  uint32_t rowoff[SLOTS];
#pragma unroll
  for (int e = 0; e < A_SLOTS; ++e) rowoff[e] = (uint32_t)min(i0 + row0 + e * ROWS_PER_PASS, a.M - 1) * a.P;
#pragma unroll
  for (int e = 0; e < B_SLOTS; ++e) rowoff[A_SLOTS + e] = (uint32_t)min(j0 + row0 + e * ROWS_PER_PASS, a.C - 1) * a.P;
  const uint32_t upar = (uint32_t)(reinterpret_cast<uintptr_t>(a.U) >> 1) & 1u;
  const uint32_t vpar = (uint32_t)(reinterpret_cast<uintptr_t>(a.V) >> 1) & 1u;
  const uint32_t* const ual = reinterpret_cast<const uint32_t*>(a.U - upar);
  const uint32_t* const val = reinterpret_cast<const uint32_t*>(a.V - vpar);

  uint32_t raw[SLOTS][5];
  uint32_t oddmask = 0u;
  uint32_t keep[4] = {~0u, ~0u, ~0u, ~0u};
  auto fetch = [&](int u) {
    const int n = u / a.slabs_per_img;
    const int sl = u - n * a.slabs_per_img;
    const int p_own = sl * kSlabK;
    const int ps = min(p_own, a.P - kSlabK);  // the last slab starts early
    const int p = ps + piece * 8;
    // pixels below p_own belong to the slab before: masked (both operands, so that nothing of them reaches a product)
    const int masked = min(8, max(0, p_own - p));
#pragma unroll
    for (int m = 0; m < 4; ++m) keep[m] = (2 * m >= masked ? 0xffffu : 0u) | (2 * m + 1 >= masked ? 0xffff0000u : 0u);
    oddmask = 0u;
    const size_t ubase = (size_t)n * a.M * a.P + p + upar, vbase = (size_t)n * a.C * a.P + p + vpar;
#pragma unroll
    for (int e = 0; e < SLOTS; ++e) {
      const size_t idx = (e < A_SLOTS ? ubase : vbase) + rowoff[e];
      const uint32_t* q = (e < A_SLOTS ? ual : val) + (idx >> 1);
      const uint32_t odd = (uint32_t)idx & 1u;
      raw[e][0] = q[0], raw[e][1] = q[1], raw[e][2] = q[2], raw[e][3] = q[3];
      raw[e][4] = q[3 + odd];  // the dword with the eighth element of a group that starts on an odd one
      oddmask |= odd << e;
    }
  };
  auto shifted = [&](int slot) -> u32x4 {
    const uint32_t odd = (oddmask >> slot) & 1u;
    const uint32_t* r = raw[slot];
    return u32x4{shift16(r[0], r[1], odd) & keep[0], shift16(r[1], r[2], odd) & keep[1], shift16(r[2], r[3], odd) & keep[2],
                 shift16(r[3], r[4], odd) & keep[3]};
  };
  auto store = [&]() {
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e)
      *reinterpret_cast<u32x4*>(As + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) = shifted(e);
#pragma unroll
    for (int e = 0; e < B_SLOTS; ++e)
      *reinterpret_cast<u32x4*>(Bs + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) = shifted(A_SLOTS + e);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  if (u0 < u1) {
    fetch(u0);
    store();
  }
  __syncthreads();
  for (int u = u0; u < u1; ++u) {
    const bool more = u + 1 < u1;
    if (more) fetch(u + 1);
#pragma unroll
    for (int i = 0; i < kSlabK / 16; ++i) {
      u32x4 af[TM], bfr[TN];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
        af[mi] = *reinterpret_cast<const u32x4*>(As + (wm0 + mi * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
        bfr[ni] = *reinterpret_cast<const u32x4*>(Bs + (wn0 + ni * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(af[mi], bfr[ni], acc[mi][ni]);
    }
    __syncthreads();  // every wave has read the slab
    if (more) store();
    __syncthreads();
  }

  float* dst = a.out + (int64_t)split * a.M * a.C;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int j = j0 + wn0 + ni * 32 + l32;
    if (j >= a.C) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row16(q, lane);
        if (i < a.M) dst[(int64_t)i * a.C + j] = acc[mi][ni][q];
      }
  }
}

// ---- host side -------------------------------------------------------------------------------------------------------
// rows: output rows of the product (maps for the forward pass, input channels for the input gradient); depth: its
// contraction length.  The kernel matrix operand is read 16 bytes at a time, so the depth must be a multiple of 8.
bool pointwise_bf16_plan(int64_t n, int64_t rows, int64_t depth, int64_t P, PointwiseBf16Plan* p) {
  if (depth % 8 != 0 || depth < 32 || rows < 32 || P < 4) return false;
  if (n * rows * P > 0x7fffffff00LL || n * depth * P > 0x7fffffff00LL) return false;
  p->bm = rows <= 64 ? 64 : 128;
  p->tiles_m = (int)ceil_div(rows, p->bm);
  p->tiles_p = (int)ceil_div(P, 128);
  return (int64_t)p->tiles_m * n * p->tiles_p <= 0x7ffffff0LL;
}

template <int BM, int BN, int WM, int WN>
static void launch_pointwise_one(const PointwiseBf16Args& a, hipStream_t st) {
  constexpr size_t lds = 2 * (size_t)(BM + BN) * kPitch * sizeof(uint16_t);
  // whole slabs, at least one pixel tile per plane, 32-bit element offsets inside the kernel matrix and a sample
  const bool fast = a.K % kSlabK == 0 && a.P >= BN && (int64_t)a.M * a.K <= 0x7fffffffLL && ((int64_t)a.K + 64) * a.P <= 0x7fffffffLL;
  auto kernel = fast ? pointwise_bf16_fast_kernel<BM, BN, WM, WN> : pointwise_bf16_kernel<BM, BN, WM, WN>;
  static bool opted[2] = {false, false};
  if (!opted[fast]) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    opted[fast] = true;
  }
  const int64_t blocks = xcd_grid((int64_t)a.tiles_m * a.n * a.tiles_p);
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kThreads), fast ? lds / 2 : lds, st, a);
}

vcnn_status launch_pointwise_bf16(const PointwiseBf16Plan& p, int n, int rows, int depth, int P, const void* A, const void* X,
                                  const float* bias, void* Y, int relu, hipStream_t st) {
  if ((reinterpret_cast<uintptr_t>(A) & 15) != 0) return fail(VCNN_ERR_UNSUPPORTED, "bf16 1x1 product: kernel matrix must be 16-byte aligned");
  PointwiseBf16Args a{};
  a.A = (const bf16*)A, a.X = (const bf16*)X, a.bias = bias, a.Y = (bf16*)Y;
  a.n = n, a.M = rows, a.K = depth, a.P = P;
  a.tiles_m = p.tiles_m, a.tiles_p = p.tiles_p, a.relu = relu;
  if (p.bm == 64)
    launch_pointwise_one<64, 128, 32, 64>(a, st);
  else
    launch_pointwise_one<128, 128, 64, 64>(a, st);
  return check_launch("pointwise_bf16");
}

// Kernel gradient: (sample, 64-pixel slab) units are dealt to blockIdx.y in contiguous runs; the partial products are
// added in ascending order by the slice sum.
bool pointwise_filter_bf16_plan(const ConvGeom& g, PointwiseFilterBf16Plan* p) {
  if (g.M < 32 || g.c < 32 || g.P < 8) return false;
  p->bm = g.M <= 64 ? 64 : 128;
  p->slabs_per_img = (int)ceil_div(g.P, kSlabK);
  const int64_t tiles = ceil_div(g.M, p->bm) * ceil_div(g.c, 128);
  const int64_t units = (int64_t)g.n * p->slabs_per_img;
  int64_t want = ceil_div(512, tiles);
  if (want > units) want = units;
  p->units_per_split = (int)ceil_div(units, want);
  p->splits = (int)ceil_div(units, p->units_per_split);
  p->partial_bytes = p->splits > 1 ? (size_t)p->splits * g.M * g.c * sizeof(float) : 0;
  return tiles * p->splits <= 0x7ffffff0LL && units <= 0x7fffffffLL;
}

template <int BM, int BN, int WM, int WN>
static void launch_pointwise_filter_one(const PointwiseFilterBf16Args& a, hipStream_t st) {
  constexpr size_t lds = 2 * (size_t)(BM + BN) * kPitch * sizeof(uint16_t);
  // at least one slab per plane, 32-bit element offsets of a row inside a sample
  const bool fast = a.P >= kSlabK && (int64_t)std::max(a.M, a.C) * a.P <= 0x7fffffffLL;
  auto kernel = fast ? pointwise_filter_bf16_fast_kernel<BM, BN, WM, WN> : pointwise_filter_bf16_kernel<BM, BN, WM, WN>;
  static bool opted[2] = {false, false};
  if (!opted[fast]) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    opted[fast] = true;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)xcd_grid((int64_t)a.tiles * a.splits)), dim3(kThreads), fast ? lds / 2 : lds, st, a);
}

vcnn_status launch_pointwise_filter_bf16(const PointwiseFilterBf16Plan& p, const ConvGeom& g, const void* x, const void* dy,
                                         float* dw, float* partial, hipStream_t st) {
  PointwiseFilterBf16Args a{};
  a.U = (const bf16*)dy, a.V = (const bf16*)x, a.out = p.splits > 1 ? partial : dw;
  a.n = g.n, a.M = (int)g.M, a.C = g.c, a.P = (int)g.P;
  a.tiles_m = (int)ceil_div(g.M, p.bm);
  a.tiles = a.tiles_m * (int)ceil_div(g.c, 128), a.splits = p.splits;
  a.slabs_per_img = p.slabs_per_img, a.units_per_split = p.units_per_split;
  if (p.bm == 64)
    launch_pointwise_filter_one<64, 128, 32, 64>(a, st);
  else
    launch_pointwise_filter_one<128, 128, 64, 64>(a, st);
  if (vcnn_status s = check_launch("pointwise_filter_bf16")) return s;
  if (p.splits == 1) return VCNN_OK;
  return launch_sum_slices(partial, nullptr, dw, VCNN_F32, g.M * g.c, p.splits, 1, 1, 0, st);
}

}  // namespace vcnn
