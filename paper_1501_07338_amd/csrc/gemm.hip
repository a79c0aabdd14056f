// Dense matrix products of the vectorized layer on the CDNA4 matrix cores (fp32 in, fp32 accumulate).
//
//   forward   (Eq. 2 / Eq. 4):  Y[M x N]    = W[M x K] * col[K x N]  (+ bias, sigma), stored as [N][M][P]
//   bwd data  (phi_c^{-1} arg): dcol[K x N] = W^T * dY
//   bwd filter:                 dW[M x K]   = dY * col^T  (contraction over the N = batch*OH*OW axis)
//   fully connected layers: the same products with plain row-major operands.
//
// All of them run v_mfma_f32_32x32x2_f32 on LDS-staged tiles.  LDS tiles are stored k-major
// ([BK][BM], [BK][BN]) so that the 32 lanes of a half-wave read 32 consecutive floats.
#include "common.h"

namespace vcnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));

static constexpr int kThreads = 256;
static constexpr int BK = 16;

__device__ __forceinline__ int64_t jmap(int j, int P, int64_t s_img, int64_t s_j) {
  if (P > 0) {
    const int q = j / P;
    return (int64_t)q * s_img + (int64_t)(j - q * P) * s_j;
  }
  return (int64_t)j * s_j;
}

// Multiply-accumulate one BK-deep pair of LDS tiles into the wave's accumulators.
// Operand layout of the 32x32x2 instruction: lane l supplies A[row l%32][k l/32] and B[k l/32][col l%32].
template <int LDA, int LDB, int TM, int TN>
__device__ __forceinline__ void mma_tile(const float* As, const float* Bs, int wm0, int wn0, int lane,
                                         f32x16 (&acc)[TM][TN]) {
  const int l32 = lane & 31;
  const int half = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < BK; kk += 2) {
    float av[TM], bv[TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) av[mi] = As[(kk + half) * LDA + wm0 + mi * 32 + l32];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) bv[ni] = Bs[(kk + half) * LDB + wn0 + ni * 32 + l32];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
  }
}

// Accumulator layout of the 32x32 result: register q of lane l holds row 8*(q/4) + 4*(l/32) + q%4, column l%32.
__device__ __forceinline__ int acc_row(int q, int lane) { return 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3); }

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(kThreads) void gemm_f32_kernel(GemmArgs a, int tiles_m) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  constexpr int LDA = BM + (A_KC ? 1 : 0);
  constexpr int LDB = BN + (B_KC ? 1 : 0);
  constexpr int NA = BM * BK / kThreads;
  constexpr int NB = BN * BK / kThreads;
  constexpr int TM = WM / 32, TN = WN / 32;
  __shared__ float As[BK * LDA];
  __shared__ float Bs[BK * LDB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int tm = blockIdx.x % tiles_m;
  const int tn = blockIdx.x / tiles_m;
  const int i0 = tm * BM;
  const int j0 = tn * BN;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;

  // Per-thread load slots.  The fastest-varying thread index walks the operand's contiguous axis.
  int a_il[NA], a_kl[NA];
  int64_t a_off[NA];
  bool a_ok[NA];
#pragma unroll
  for (int e = 0; e < NA; ++e) {
    if (A_KC) {
      a_kl[e] = tid % BK;
      a_il[e] = tid / BK + e * (kThreads / BK);
    } else {
      a_il[e] = tid % BM;
      a_kl[e] = tid / BM + e * (kThreads / BM);
    }
    a_ok[e] = (i0 + a_il[e]) < a.M;
    a_off[e] = (int64_t)(i0 + a_il[e]) * a.a_si + (int64_t)a_kl[e] * a.a_sk;
  }
  int b_jl[NB], b_kl[NB];
  int64_t b_off[NB];
  bool b_ok[NB];
#pragma unroll
  for (int e = 0; e < NB; ++e) {
    if (B_KC) {
      b_kl[e] = tid % BK;
      b_jl[e] = tid / BK + e * (kThreads / BK);
    } else {
      b_jl[e] = tid % BN;
      b_kl[e] = tid / BN + e * (kThreads / BN);
    }
    const int j = j0 + b_jl[e];
    b_ok[e] = j < a.N;
    b_off[e] = (b_ok[e] ? jmap(j, a.b_P, a.b_simg, a.b_sj) : 0) + (int64_t)b_kl[e] * a.b_sk;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  float ra[NA], rb[NB];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int e = 0; e < NA; ++e)
      ra[e] = (a_ok[e] && (k0 + a_kl[e]) < a.K) ? a.A[a_off[e] + (int64_t)k0 * a.a_sk] : 0.f;
#pragma unroll
    for (int e = 0; e < NB; ++e)
      rb[e] = (b_ok[e] && (k0 + b_kl[e]) < a.K) ? a.B[b_off[e] + (int64_t)k0 * a.b_sk] : 0.f;
  };

  const int ktiles = (a.K + BK - 1) / BK;
  fetch(0);
  for (int kt = 0; kt < ktiles; ++kt) {
#pragma unroll
    for (int e = 0; e < NA; ++e) As[a_kl[e] * LDA + a_il[e]] = ra[e];
#pragma unroll
    for (int e = 0; e < NB; ++e) Bs[b_kl[e] * LDB + b_jl[e]] = rb[e];
    __syncthreads();
    if (kt + 1 < ktiles) fetch((kt + 1) * BK);
    mma_tile<LDA, LDB, TM, TN>(As, Bs, wm0, wn0, lane, acc);
    __syncthreads();
  }

  const int l32 = lane & 31;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int j = j0 + wn0 + ni * 32 + l32;
    if (j >= a.N) continue;
    const int64_t cj = jmap(j, a.c_P, a.c_simg, a.c_sj);
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row(q, lane);
        if (i < a.M) {
          float v = acc[mi][ni][q];
          if (a.bias) v += a.bias[i];
          if (a.relu) v = fmaxf(v, 0.f);
          a.C[(int64_t)i * a.c_si + cj] = v;
        }
      }
  }
}

template <int BM, int BN, int WM, int WN>
static void launch_cfg(const GemmArgs& a, bool a_kc, bool b_kc, hipStream_t st) {
  const int tiles_m = (int)ceil_div(a.M, BM);
  const int64_t blocks = (int64_t)tiles_m * ceil_div(a.N, BN);
  const dim3 grid((unsigned)blocks), block(kThreads);
  if (a_kc && b_kc)
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, true, true>), grid, block, 0, st, a, tiles_m);
  else if (a_kc)
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, true, false>), grid, block, 0, st, a, tiles_m);
  else if (b_kc)
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, false, true>), grid, block, 0, st, a, tiles_m);
  else
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, WM, WN, false, false>), grid, block, 0, st, a, tiles_m);
}

vcnn_status launch_gemm_f32(const GemmArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(VCNN_ERR_SHAPE, "gemm: empty operand");
  const bool a_kc = (a.a_sk == 1) && (a.a_si != 1);
  const bool b_kc = (a.b_sk == 1) && (a.b_sj != 1);
  if (a.M <= 32)
    launch_cfg<32, 256, 32, 64>(a, a_kc, b_kc, st);
  else if (a.M <= 64)
    launch_cfg<64, 256, 64, 64>(a, a_kc, b_kc, st);
  else
    launch_cfg<128, 128, 64, 64>(a, a_kc, b_kc, st);
  return check_launch("gemm_f32");
}

// -------------------------------------------------------------------------------------------------
// Filter gradient: dW[m][k] = sum_j dY(m, j) * col[k][j].  Both operands are contiguous along the
// contraction index j; dY lives in [N][M][P] layout, so j = n*P + p addresses dy[(n*M + m)*P + p].
// blockIdx.y selects a range of columns; each range writes its own partial product and a second
// kernel adds the partials in ascending order, which keeps the result independent of scheduling.
// -------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void bwd_filter_f32_kernel(ConvGeom g, const float* __restrict__ dy,
                                                                  const float* __restrict__ col,
                                                                  float* __restrict__ out, int tiles_m, int chunk) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  constexpr int LDA = BM + 1, LDB = BN + 1;
  constexpr int NA = BM * BK / kThreads, NB = BN * BK / kThreads;
  constexpr int TM = WM / 32, TN = WN / 32;
  __shared__ float As[BK * LDA];
  __shared__ float Bs[BK * LDB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int i0 = tm * BM, k0 = tn * BN;  // i: output map (row of dW); k: patch-matrix row (column of dW)
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int64_t js = (int64_t)blockIdx.y * chunk;
  const int64_t je = min((int64_t)g.N, js + chunk);
  const int M = (int)g.M, K = (int)g.K;
  const int P = (int)g.P;

  const int kl = tid % BK;       // position along the contraction axis inside a BK slab
  const int rl = tid / BK;       // first tile row this thread loads; further rows at +16
  // (n, p) of this thread's first contraction index.
  int64_t j = js + kl;
  int n = (int)(j / P);
  int p = (int)(j - (int64_t)n * P);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  float ra[NA], rb[NB];
  auto fetch = [&]() {
    const bool jin = j < je;
#pragma unroll
    for (int e = 0; e < NA; ++e) {
      const int m = i0 + rl + e * (kThreads / BK);
      ra[e] = (jin && m < M) ? dy[((int64_t)n * M + m) * P + p] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < NB; ++e) {
      const int k = k0 + rl + e * (kThreads / BK);
      rb[e] = (jin && k < K) ? col[(int64_t)k * g.N + j] : 0.f;
    }
    j += BK;
    p += BK;
    while (p >= P) {
      p -= P;
      ++n;
    }
  };

  const int ktiles = (int)((je - js + BK - 1) / BK);
  if (ktiles > 0) fetch();
  for (int kt = 0; kt < ktiles; ++kt) {
#pragma unroll
    for (int e = 0; e < NA; ++e) As[kl * LDA + rl + e * (kThreads / BK)] = ra[e];
#pragma unroll
    for (int e = 0; e < NB; ++e) Bs[kl * LDB + rl + e * (kThreads / BK)] = rb[e];
    __syncthreads();
    if (kt + 1 < ktiles) fetch();
    mma_tile<LDA, LDB, TM, TN>(As, Bs, wm0, wn0, lane, acc);
    __syncthreads();
  }

  float* dst = out + (int64_t)blockIdx.y * M * K;
  const int l32 = lane & 31;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int k = k0 + wn0 + ni * 32 + l32;
    if (k >= K) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int m = i0 + wm0 + mi * 32 + acc_row(q, lane);
        if (m < M) dst[(int64_t)m * K + k] = acc[mi][ni][q];
      }
  }
}

__global__ __launch_bounds__(kThreads) void sum_partials_kernel(const float* __restrict__ partial,
                                                                float* __restrict__ out, int64_t count, int splits) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= count) return;
  float acc = 0.f;
  for (int s = 0; s < splits; ++s) acc += partial[(int64_t)s * count + i];
  out[i] = acc;
}

static int bwd_filter_bm(const ConvGeom& g) { return g.M <= 32 ? 32 : (g.M <= 64 ? 64 : 128); }
static int bwd_filter_bn(const ConvGeom& g) { return g.M <= 64 ? 128 : 128; }

static int bwd_filter_chunk(const ConvGeom& g) {
  const int64_t tiles = ceil_div(g.M, bwd_filter_bm(g)) * ceil_div(g.K, bwd_filter_bn(g));
  int64_t want = 1024 / tiles;
  const int64_t max_splits = g.N / 512 > 0 ? g.N / 512 : 1;
  if (want < 1) want = 1;
  if (want > max_splits) want = max_splits;
  int64_t chunk = ceil_div(g.N, want);
  chunk = ceil_div(chunk, BK) * BK;
  return (int)chunk;
}

int bwd_filter_splits(const ConvGeom& g) { return (int)ceil_div(g.N, bwd_filter_chunk(g)); }

size_t bwd_filter_partial_bytes(const ConvGeom& g) {
  const int splits = bwd_filter_splits(g);
  return splits > 1 ? (size_t)splits * g.M * g.K * sizeof(float) : 0;
}

vcnn_status launch_bwd_filter_gemm_f32(const ConvGeom& g, const float* dy, const float* col, float* dw,
                                       float* partial, hipStream_t st) {
  const int chunk = bwd_filter_chunk(g);
  const int splits = bwd_filter_splits(g);
  float* out = splits > 1 ? partial : dw;
  const int bm = bwd_filter_bm(g);
  const int tiles_m = (int)ceil_div(g.M, bm);
  const int64_t tiles = (int64_t)tiles_m * ceil_div(g.K, bwd_filter_bn(g));
  const dim3 grid((unsigned)tiles, (unsigned)splits), block(kThreads);
  if (splits > 65535) return fail(VCNN_ERR_UNSUPPORTED, "bwd_filter: too many contraction splits");
  if (bm == 32)
    hipLaunchKernelGGL((bwd_filter_f32_kernel<32, 128, 32, 32>), grid, block, 0, st, g, dy, col, out, tiles_m, chunk);
  else if (bm == 64)
    hipLaunchKernelGGL((bwd_filter_f32_kernel<64, 128, 32, 64>), grid, block, 0, st, g, dy, col, out, tiles_m, chunk);
  else
    hipLaunchKernelGGL((bwd_filter_f32_kernel<128, 128, 64, 64>), grid, block, 0, st, g, dy, col, out, tiles_m, chunk);
  vcnn_status s = check_launch("bwd_filter_f32");
  if (s != VCNN_OK || splits == 1) return s;
  const int64_t count = g.M * g.K;
  hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)ceil_div(count, kThreads)), block, 0, st, partial, dw, count,
                     splits);
  return check_launch("sum_partials");
}

}  // namespace vcnn
