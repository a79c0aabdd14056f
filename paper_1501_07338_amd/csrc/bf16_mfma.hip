// bfloat16 matrix-core kernels (v_mfma_f32_32x32x16_bf16: 16 contraction steps per instruction, fp32
// accumulate) for the bf16 variant of the layer path.
//
//  * conv_halo_bf16_kernel: implicit-unroll convolution.  As in the fp32 kernel the patch matrix is
//    never formed: input rows (+ halo) are staged in LDS and the B operand is read at
//    lane_base(pixel) + tap_offset.  A lane's B operand is 8 consecutive contraction indices, so the
//    contraction is ordered (channel group of 8, r, s, channel in group) and the LDS tile keeps the 8
//    channels of a group interleaved: one 16-byte LDS read per operand.  The kernel matrix is
//    re-ordered to match by reorder_weights_kernel (which also flips / transposes it for the input
//    gradient); padding channels carry zero weights.
//  * gemm_nt_bf16_kernel: C[M x N] = A[M x K] * B[N x K]^T with both operands contraction-contiguous,
//    contraction split over blockIdx.y.  Used for the filter gradient dW = dY * phi_c(x)^T on the bf16
//    patch matrix, with dY first re-laid as [M][batch*P] by repack_dy_kernel.
#include <algorithm>

#include "common.h"
#include "elem.h"

namespace vcnn {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr int kThreads = 256;
static constexpr int kSlabK = 64;            // contraction elements per LDS slab
static constexpr int kPitch = kSlabK + 8;    // bf16 elements per LDS row (16-byte aligned, conflict-spreading)
static constexpr size_t kLdsBudget = 78 * 1024;

__device__ __forceinline__ f32x16 mfma_bf16(uint4 a, uint4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ int acc_row16(int q, int lane) { return 8 * (q >> 2) + 4 * (lane >> 5) + (q & 3); }

// ---- kernel-matrix re-ordering ---------------------------------------------------------------------------
// out[o][g][q][c8] = in[o*so + (8g+c8)*si + (flip ? RS-1-q : q)]  for 8g+c8 < CI, else 0.
__global__ __launch_bounds__(kThreads) void reorder_weights_kernel(const bf16* __restrict__ in, bf16* __restrict__ out,
                                                                   int CO, int CI, int RS, int64_t so, int64_t si,
                                                                   int flip) {
  const int CG = (CI + 7) / 8;
  const int64_t total = (int64_t)CO * CG * RS * 8;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= total) return;
  const int c8 = (int)(i & 7);
  int64_t t = i >> 3;
  const int q = (int)(t % RS);
  t /= RS;
  const int g = (int)(t % CG);
  const int o = (int)(t / CG);
  const int c = g * 8 + c8;
  bf16 v;
  v.bits = 0;
  if (c < CI) v = in[(int64_t)o * so + (int64_t)c * si + (flip ? RS - 1 - q : q)];
  out[i] = v;
}

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

// ---- implicit-unroll convolution -------------------------------------------------------------------------
struct HaloBf16Args {
  const bf16* x;      // [n][c][h][w]
  const bf16* wre;    // [m][cg][rs][8]  re-ordered kernel matrix
  const float* bias;  // [m] or null
  bf16* y;            // [n][m][oh][ow]
  int n, c, h, w, m, r, s, ph, pw, oh, ow, P;
  int tiles_m, tiles_per_img;
  int cg;             // channel groups of 8 (total)
  int cgc;            // channel groups staged per chunk
  int nr, wp;         // halo rows and row pitch (positions) per group
  int uch;            // (group, tap) pairs per full chunk, padded to a multiple of 8
  int relu;
};

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void conv_halo_bf16_kernel(HaloBf16Args a) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_SLAB = BM * kPitch;  // bf16 elements
  extern __shared__ uint4 smem16[];
  bf16* const As0 = reinterpret_cast<bf16*>(smem16);                  // 2 slabs [BM][kPitch]
  int* const tbl = reinterpret_cast<int*>(As0 + 2 * A_SLAB);          // [uch] de-interleaved per slab: [slab][half][4]
  uint4* const halo = reinterpret_cast<uint4*>(tbl + a.uch);          // [cgc][nr][wp] positions of 8 channels

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int tm = blockIdx.x % a.tiles_m;
  const int tj = blockIdx.x / a.tiles_m;
  const int n = tj / a.tiles_per_img;
  const int p0 = (tj - n * a.tiles_per_img) * BN;
  const int i0 = tm * BM;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int RS = a.r * a.s;
  const int plane = a.nr * a.wp;
  const int oh_first = p0 / a.ow;
  const int64_t wrow = (int64_t)a.cg * RS * 8;  // elements per row of the re-ordered kernel matrix

  // table: position offset of pair u = (group gl, tap q) inside the halo tile; padding pairs point at 0
  // (their kernel-matrix entries are zero).  Entry u = 8*sl + 2*i + h is stored at 8*sl + 4*h + i.
  for (int u = tid; u < a.uch; u += kThreads) {
    int off = 0;
    if (u < a.cgc * RS) {
      const int gl = u / RS;
      const int q = u - gl * RS;
      const int r = q / a.s;
      off = gl * plane + r * a.wp + (q - r * a.s);
    }
    const int sl = u >> 3, w8 = u & 7;
    tbl[sl * 8 + (w8 & 1) * 4 + (w8 >> 1)] = off;
  }

  int lane_base[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = min(p0 + wn0 + ni * 32 + l32, a.P - 1);
    const int oh = p / a.ow;
    lane_base[ni] = (oh - oh_first) * a.wp + (p - oh * a.ow);
  }

  // kernel-matrix staging: thread -> (row, 16-byte piece of the 64-element slab)
  constexpr int ROWS_PER_PASS = kThreads / 8;
  constexpr int A_SLOTS = BM / ROWS_PER_PASS;
  const int piece = tid & 7, row0 = tid >> 3;
  uint4 areg[A_SLOTS];
  bool a_ok[A_SLOTS];

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  const bf16* xin = a.x + (int64_t)n * a.c * a.h * a.w;

  for (int g0 = 0; g0 < a.cg; g0 += a.cgc) {
    const int cgc = min(a.cgc, a.cg - g0);
    const int ulen = cgc * RS;               // valid (group, tap) pairs in this chunk
    const int64_t ubase = (int64_t)g0 * RS;  // first pair of the chunk in the re-ordered matrix
    auto fetch = [&](int sl) {
      const int u = sl * 8 + piece;
#pragma unroll
      for (int e = 0; e < A_SLOTS; ++e) {
        const int m = i0 + row0 + e * ROWS_PER_PASS;
        a_ok[e] = m < a.m && u < ulen;
        const bf16* src = a.wre + (int64_t)min(m, a.m - 1) * wrow + (ubase + min(u, ulen - 1)) * 8;
        areg[e] = *reinterpret_cast<const uint4*>(src);
      }
    };
    auto store = [&](bf16* As) {
#pragma unroll
      for (int e = 0; e < A_SLOTS; ++e)
        *reinterpret_cast<uint4*>(As + (row0 + e * ROWS_PER_PASS) * kPitch + piece * 8) =
            a_ok[e] ? areg[e] : make_uint4(0u, 0u, 0u, 0u);
    };
    fetch(0);
    __syncthreads();  // the previous chunk's MFMAs are done with the halo tile and the slabs
    // stage the input rows of this chunk, 8 channels interleaved per position, zero padded
    {
      uint16_t* h16 = reinterpret_cast<uint16_t*>(halo);
      const int lines = cgc * 8 * a.nr;  // (group, channel in group, row)
      for (int line = wave; line < lines; line += kThreads / 64) {
        const int ry = line % a.nr;
        const int cl = line / a.nr;  // gl*8 + c8
        const int gl = cl >> 3, c8 = cl & 7;
        const int c = (g0 + gl) * 8 + c8;
        const int ih = oh_first - a.ph + ry;
        const bool row_ok = c < a.c && ih >= 0 && ih < a.h;
        const bf16* src = xin + ((int64_t)(row_ok ? c : 0) * a.h + (row_ok ? ih : 0)) * a.w;
        uint16_t* dst = h16 + ((int64_t)(gl * a.nr + ry) * a.wp) * 8 + c8;
        for (int rx = lane; rx < a.wp; rx += 64) {
          const int iw = rx - a.pw;
          const bool ok = row_ok && iw >= 0 && iw < a.w;
          const uint16_t v = src[ok ? iw : 0].bits;
          dst[rx * 8] = ok ? v : (uint16_t)0;
        }
      }
    }
    store(As0);
    __syncthreads();

    const int slabs = (ulen + 7) >> 3;
    for (int sl = 0; sl < slabs; ++sl) {
      const int cur = sl & 1;
      const bool more = sl + 1 < slabs;
      if (more) fetch(sl + 1);
      const bf16* As = As0 + cur * A_SLAB;
      const int4 o4 = *reinterpret_cast<const int4*>(tbl + sl * 8 + half * 4);
      const int o[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint4 af[TM], bfr[TN];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
          af[mi] = *reinterpret_cast<const uint4*>(As + (wm0 + mi * 32 + l32) * kPitch + (2 * i + half) * 8);
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) bfr[ni] = halo[lane_base[ni] + o[i]];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(af[mi], bfr[ni], acc[mi][ni]);
      }
      if (more) store(As0 + (cur ^ 1) * A_SLAB);
      __syncthreads();
    }
  }

#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = p0 + wn0 + ni * 32 + l32;
    if (p >= a.P) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row16(q, lane);
        if (i < a.m) {
          float v = acc[mi][ni][q];
          if (a.bias) v += a.bias[i];
          if (a.relu) v = fmaxf(v, 0.f);
          st(a.y + ((int64_t)n * a.m + i) * a.P + p, v);
        }
      }
  }
}

size_t reordered_weight_bytes(int co, int ci, int rs) { return (size_t)co * ((ci + 7) / 8) * rs * 8 * sizeof(uint16_t); }

bool conv_halo_bf16_plan(int n, int c, int h, int w, int m, int r, int s, int ph, int pw, HaloBf16Plan* p) {
  const int oh = h + 2 * ph - r + 1, ow = w + 2 * pw - s + 1;
  if (oh <= 0 || ow <= 0) return false;
  const int bm = m <= 32 ? 32 : (m <= 64 ? 64 : 128);
  const int bn = m <= 64 ? 256 : 128;
  const int rs = r * s;
  const int cg = (c + 7) / 8;
  int rows = (bn + ow - 2) / ow + 1;
  if (rows > oh) rows = oh;
  const int nr = rows + r - 1, wp = w + 2 * pw;
  const size_t a_bytes = 2 * (size_t)bm * kPitch * sizeof(uint16_t);
  int best = 0;
  for (int cgc = 1; cgc <= cg; ++cgc) {
    const int uch = (int)ceil_div((int64_t)cgc * rs, 8) * 8;
    const size_t bytes = a_bytes + (size_t)uch * 4 + (size_t)cgc * nr * wp * 16;
    if (bytes > kLdsBudget || uch > 4096) break;
    best = cgc;
  }
  if (best == 0) return false;
  // among chunk sizes at least half the largest, take the one that pads the fewest (group, tap) pairs
  int pick = best;
  double pick_waste = 2.0;
  for (int cgc = best; cgc >= 1 && 2 * cgc > best; --cgc) {
    const int64_t chunks = ceil_div(cg, cgc);
    const int last = cg - (int)(chunks - 1) * cgc;
    const int64_t slabs = (chunks - 1) * ceil_div((int64_t)cgc * rs, 8) + ceil_div((int64_t)last * rs, 8);
    const double waste = 1.0 - (double)cg * rs / (double)(slabs * 8);
    if (waste < pick_waste - 1e-9) pick = cgc, pick_waste = waste;
  }
  p->bm = bm, p->bn = bn, p->cg = cg, p->cgc = pick, p->nr = nr, p->wp = wp;
  p->uch = (int)ceil_div((int64_t)pick * rs, 8) * 8;
  p->lds_bytes = a_bytes + (size_t)p->uch * 4 + (size_t)pick * nr * wp * 16;
  const int64_t tiles = ceil_div(m, bm) * (int64_t)n * ceil_div((int64_t)oh * ow, bn);
  return tiles <= 0x7fffffffLL;
}

vcnn_status launch_reorder_weights(const void* w, void* out, int co, int ci, int rs, int64_t so, int64_t si, int flip,
                                   hipStream_t st) {
  const int64_t total = (int64_t)co * ((ci + 7) / 8) * rs * 8;
  hipLaunchKernelGGL(reorder_weights_kernel, dim3((unsigned)ceil_div(total, kThreads)), dim3(kThreads), 0, st,
                     (const bf16*)w, (bf16*)out, co, ci, rs, so, si, flip);
  return check_launch("reorder_weights");
}

template <int BM, int BN, int WM, int WN>
static void launch_halo_bf16(const HaloBf16Args& a, const HaloBf16Plan& p, hipStream_t st) {
  const dim3 grid((unsigned)((int64_t)a.tiles_m * a.n * a.tiles_per_img)), block(kThreads);
  auto kernel = conv_halo_bf16_kernel<BM, BN, WM, WN>;
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsBudget);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, st, a);
}

vcnn_status launch_conv_halo_bf16(const HaloBf16Plan& p, int n, int c, int h, int w, int m, int r, int s, int ph, int pw,
                                  const void* x, const void* wre, const float* bias, void* y, int relu, hipStream_t st) {
  HaloBf16Args a{};
  a.x = (const bf16*)x, a.wre = (const bf16*)wre, a.bias = bias, a.y = (bf16*)y;
  a.n = n, a.c = c, a.h = h, a.w = w, a.m = m, a.r = r, a.s = s, a.ph = ph, a.pw = pw;
  a.oh = h + 2 * ph - r + 1, a.ow = w + 2 * pw - s + 1;
  a.P = a.oh * a.ow;
  a.tiles_m = (int)ceil_div(m, p.bm);
  a.tiles_per_img = (int)ceil_div(a.P, p.bn);
  a.cg = p.cg, a.cgc = p.cgc, a.nr = p.nr, a.wp = p.wp, a.uch = p.uch, a.relu = relu;
  if (p.bm == 32)
    launch_halo_bf16<32, 256, 32, 64>(a, p, st);
  else if (p.bm == 64)
    launch_halo_bf16<64, 256, 64, 64>(a, p, st);
  else
    launch_halo_bf16<128, 128, 64, 64>(a, p, st);
  return check_launch("conv_halo_bf16");
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
