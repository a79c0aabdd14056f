// bfloat16 matrix-core product (v_mfma_f32_32x32x16_bf16: 16 contraction steps per instruction, fp32
// accumulate) for the filter gradient of the bf16 variant.
//
// gemm_nt_bf16_kernel: C[M x N] = A[M x K] * B[N x K]^T with both operands contraction-contiguous,
// contraction split over blockIdx.y.  Used for dW = dY * phi_c(x)^T on the bf16 patch matrix, with dY
// first re-laid as [M][batch*P] by repack_dy_kernel.
#include <algorithm>

#include "common.h"
#include "elem.h"

namespace vcnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr int kThreads = 256;
static constexpr int kSlabK = 64;            // contraction elements per LDS slab
static constexpr int kPitch = kSlabK + 8;    // bf16 elements per LDS row (16-byte aligned, conflict-spreading)

__device__ __forceinline__ f32x16 mfma_bf16(uint4 a, uint4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ int acc_row16(int q, int lane) { return 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3); }

// dyt[m][n*P + p] = dy[n][m][p]
__global__ __launch_bounds__(kThreads) void repack_dy_kernel(const bf16* __restrict__ dy, bf16* __restrict__ dyt, int N,
                                                             int M, int P) {
  const int64_t total = (int64_t)N * M * P;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= total) return;
  const int p = (int)(i % P);
  const int64_t t = i / P;
  const int m = (int)(t % M);
  const int n = (int)(t / M);
  dyt[(int64_t)m * N * P + (int64_t)n * P + p] = dy[i];
}

// ---- C = A * B^T, both operands contraction-contiguous ---------------------------------------------------
struct GemmNtArgs {
  const bf16* A;  // [M][lda]
  const bf16* B;  // [N][ldb]
  float* C;       // [splits][M][N]
  int M, N;
  int64_t K, lda, ldb;
  int tiles_m;
  int64_t chunk;  // contraction elements per split (multiple of kSlabK)
};

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void gemm_nt_bf16_kernel(GemmNtArgs a) {
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
  const int i0 = (blockIdx.x % a.tiles_m) * BM;
  const int j0 = (blockIdx.x / a.tiles_m) * BN;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int64_t ks = (int64_t)blockIdx.y * a.chunk;
  const int64_t ke = min(a.K, ks + a.chunk);
  const int piece = tid & 7, row0 = tid >> 3;

  uint4 areg[A_SLOTS], breg[B_SLOTS];
  bool aok[A_SLOTS], bok[B_SLOTS];
  auto fetch = [&](int64_t k0) {
    const int64_t k = k0 + piece * 8;
    const bool kin = k < ke;  // K and the chunk are multiples of 8: a piece is inside or outside as a whole
    const int64_t kk = kin ? k : ks;
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e) {
      const int i = i0 + row0 + e * ROWS_PER_PASS;
      aok[e] = kin && i < a.M;
      areg[e] = *reinterpret_cast<const uint4*>(a.A + (int64_t)min(i, a.M - 1) * a.lda + kk);
    }
#pragma unroll
    for (int e = 0; e < B_SLOTS; ++e) {
      const int j = j0 + row0 + e * ROWS_PER_PASS;
      bok[e] = kin && j < a.N;
      breg[e] = *reinterpret_cast<const uint4*>(a.B + (int64_t)min(j, a.N - 1) * a.ldb + kk);
    }
  };
  auto store = [&](bf16* As, bf16* Bs) {
#pragma unroll
    for (int e = 0; e < A_SLOTS; ++e)
      *reinterpret_cast<uint4*>(As + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) =
          aok[e] ? areg[e] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int e = 0; e < B_SLOTS; ++e)
      *reinterpret_cast<uint4*>(Bs + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) =
          bok[e] ? breg[e] : make_uint4(0u, 0u, 0u, 0u);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  const int slabs = (int)((ke - ks + kSlabK - 1) / kSlabK);
  if (slabs > 0) {
    fetch(ks);
    store(As0, Bs0);
  }
  __syncthreads();
  for (int sl = 0; sl < slabs; ++sl) {
    const int cur = sl & 1;
    const bool more = sl + 1 < slabs;
    if (more) fetch(ks + (int64_t)(sl + 1) * kSlabK);
    const bf16* As = As0 + cur * A_SLAB;
    const bf16* Bs = Bs0 + cur * B_SLAB;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint4 af[TM], bfr[TN];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
        af[mi] = *reinterpret_cast<const uint4*>(As + (wm0 + mi * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
        bfr[ni] = *reinterpret_cast<const uint4*>(Bs + (wn0 + ni * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(af[mi], bfr[ni], acc[mi][ni]);
    }
    if (more) store(As0 + (cur ^ 1) * A_SLAB, Bs0 + (cur ^ 1) * B_SLAB);
    __syncthreads();
  }

  float* dst = a.C + (int64_t)blockIdx.y * a.M * a.N;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int j = j0 + wn0 + ni * 32 + l32;
    if (j >= a.N) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row16(q, lane);
        if (i < a.M) dst[(int64_t)i * a.N + j] = acc[mi][ni][q];
      }
  }
}

// Filter gradient in the bf16 variant: dW[M][K] = dYt[M][N] * col[K][N]^T.
bool bwd_filter_bf16_plan(const ConvGeom& g, BwdFilterBf16Plan* p) {
  if (g.N % 8 != 0 || g.M < 32) return false;
  p->bm = g.M <= 32 ? 32 : (g.M <= 64 ? 64 : 128);
  const int64_t tiles = ceil_div(g.M, p->bm) * ceil_div(g.K, 128);
  int64_t want = ceil_div(1024, tiles);
  const int64_t max_splits = std::max<int64_t>(1, g.N / 1024);
  if (want > max_splits) want = max_splits;
  int64_t chunk = ceil_div(ceil_div(g.N, want), kSlabK) * kSlabK;
  p->chunk = chunk;
  p->splits = (int)ceil_div(g.N, chunk);
  p->dyt_bytes = ((size_t)g.M * g.N * 2 + 255) & ~(size_t)255;
  p->col_bytes = ((size_t)g.K * g.N * 2 + 255) & ~(size_t)255;
  p->partial_bytes = p->splits > 1 ? (size_t)p->splits * g.M * g.K * sizeof(float) : 0;
  return p->splits <= 65535 && tiles <= 0x7fffffffLL;
}

template <int BM, int BN, int WM, int WN>
static void launch_nt(const GemmNtArgs& a, int splits, hipStream_t st) {
  const int64_t tiles = (int64_t)a.tiles_m * ceil_div(a.N, BN);
  constexpr size_t lds = 2 * (size_t)(BM + BN) * kPitch * sizeof(uint16_t);
  auto kernel = gemm_nt_bf16_kernel<BM, BN, WM, WN>;
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)tiles, (unsigned)splits), dim3(kThreads), lds, st, a);
}

vcnn_status launch_bwd_filter_bf16(const BwdFilterBf16Plan& p, const ConvGeom& g, const void* x, const void* dy, float* dw,
                                   void* workspace, hipStream_t st) {
  bf16* dyt = (bf16*)workspace;
  bf16* col = (bf16*)((char*)workspace + p.dyt_bytes);
  float* partial = (float*)((char*)workspace + p.dyt_bytes + p.col_bytes);
  const int64_t total = (int64_t)g.M * g.N;
  hipLaunchKernelGGL(repack_dy_kernel, dim3((unsigned)ceil_div(total, kThreads)), dim3(kThreads), 0, st, (const bf16*)dy,
                     dyt, g.n, (int)g.M, (int)g.P);
  if (vcnn_status s = check_launch("repack_dy")) return s;
  if (vcnn_status s = launch_im2col(g, VCNN_BF16, x, col, st)) return s;
  GemmNtArgs a{};
  a.A = dyt, a.B = col, a.C = p.splits > 1 ? partial : dw;
  a.M = (int)g.M, a.N = (int)g.K, a.K = g.N, a.lda = g.N, a.ldb = g.N;
  a.tiles_m = (int)ceil_div(g.M, p.bm);
  a.chunk = p.chunk;
  if (p.bm == 32)
    launch_nt<32, 128, 32, 32>(a, p.splits, st);
  else if (p.bm == 64)
    launch_nt<64, 128, 32, 64>(a, p.splits, st);
  else
    launch_nt<128, 128, 64, 64>(a, p.splits, st);
  if (vcnn_status s = check_launch("gemm_nt_bf16")) return s;
  if (p.splits == 1) return VCNN_OK;
  return launch_sum_slices(partial, nullptr, dw, VCNN_F32, g.M * g.K, p.splits, 1, 1, 0, st);
}

}  // namespace vcnn
