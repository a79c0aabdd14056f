// Implicit-unroll convolution on the matrix cores: the patch matrix phi_c(x) of Eq. 2 / Eq. 4 is never
// written.  A block owns BM output maps x BN output pixels of one sample (a run of consecutive pixels, or - for
// tall kernels on wide planes - a strip of rows x columns).  For a chunk of
// input channels it stages the input rows those pixels touch (with their halo, zero padded) in LDS;
// the B operand of every MFMA step is then read straight from that tile at
//     lane_base(pixel) + tap_offset(c, r, s),
// i.e. the column of the patch matrix is formed by address arithmetic at the moment it is consumed.
// The kernel matrix (A operand) streams through double-buffered LDS slabs exactly as in the plain
// product.  Each input element is fetched from global memory once per block and reused R*S*BM times.
//
// The same kernel computes the input gradient (phi_c^{-1} of the transposed product, evaluated in
// gather form): dx is the correlation of dy with the flipped, channel-transposed kernels, which a small
// kernel writes to the workspace first.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "elem.h"
#include "mma_core.h"

namespace vcnn {

static constexpr int kThreads = 256;

struct HaloArgs {
  const void* x;      // [n][c][h][w]       element type T (float or bf16)
  const void* wgt;    // [m][c*r*s]         element type T
  const float* bias;  // [m] or null
  void* y;            // [n][m][oh][ow]     element type T
  int n, c, h, w, m, r, s, ph, pw, oh, ow;
  int P;              // oh*ow
  int tiles_m, tiles_per_img;
  int cc;             // channels per chunk
  int nr;             // halo rows per channel tile
  int wp;             // halo row pitch (w + 2*pw)
  int kch;            // taps per full chunk, padded to a multiple of BK
  int relu;
  int tw, tiles_x;    // tw > 0: a tile is a strip of BN / tw output rows x tw output columns (tiles_x strips side by side)
};

// Pixel q of a block's tile as a flat index into the sample's output plane (-1: outside it), and its position inside
// the halo tile.  Tiles are runs of consecutive pixels starting at p0 (first row oh0), or strips whose first pixel is
// (oh0, ow0).  A pixel outside the plane still gets a position inside the tile: its products are dropped at the end.
__device__ __forceinline__ int tile_pixel(const HaloArgs& a, int p0, int oh0, int ow0, int q, int* base) {
  if (a.tw) {
    const int ty = q / a.tw, tx = q - ty * a.tw;
    *base = ty * a.wp + tx;
    const int oh = oh0 + ty, ow = ow0 + tx;
    return oh < a.oh && ow < a.ow ? oh * a.ow + ow : -1;
  }
  const int p = min(p0 + q, a.P - 1);
  const int oh = p / a.ow;
  *base = (oh - oh0) * a.wp + (p - oh * a.ow);
  return p0 + q < a.P ? p : -1;
}

// Copies channels [0, cc) x rows ih0 + [0, nr) x columns -pw + [0, wp) of one sample's planes x[.][h][w]
// into the LDS tile [cc][nr][wp]; positions outside the image, and channels at or beyond cvalid, become
// zero.  Elements are taken in flat tile order so every thread stays busy whatever the row length, and
// each thread issues U global loads before it stores any of them (the loads overlap their latencies).
template <int U, typename T>
__device__ __forceinline__ void stage_halo(float* halo, const T* x, int cc, int cvalid, int nr, int wp, int h, int w,
                                           int ih0, int pw, int tid) {
  const int total = cc * nr * wp;
  const int dq = kThreads / wp, dr = kThreads - dq * wp;
  int row = tid / wp;
  int rx = tid - row * wp;
  int cl = row / nr;
  int ry = row - cl * nr;
  for (int e0 = tid; e0 < total; e0 += U * kThreads) {
    float v[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ih = ih0 + ry, iw = rx - pw;
      ok[u] = e0 + u * kThreads < total && cl < cvalid && ih >= 0 && ih < h && iw >= 0 && iw < w;
      v[u] = ld(x + (ok[u] ? (cl * h + ih) * w + iw : 0));
      rx += dr;
      ry += dq;
      if (rx >= wp) rx -= wp, ++ry;
      while (ry >= nr) ry -= nr, ++cl;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (e0 + u * kThreads < total) halo[e0 + u * kThreads] = ok[u] ? v[u] : 0.f;
  }
}

template <int BM, int BN, int WM, int WN, int BK, bool VEC, typename T>
__global__ __launch_bounds__(kThreads) void conv_halo_kernel(HaloArgs a) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  using LA = LdsTile<BM, BK, true>;
  using SA = Stager<BM, BK, kThreads, true, VEC>;
  constexpr int TM = WM / 32, TN = WN / 32;
  extern __shared__ float4 smem4[];
  float* const As0 = reinterpret_cast<float*>(smem4);       // 2 slabs of the kernel matrix
  int* const tapoff = reinterpret_cast<int*>(As0 + 2 * LA::SIZE);  // [kch]
  float* const halo = As0 + 2 * LA::SIZE + a.kch;           // [cc][nr][wp]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int tm = blockIdx.x % a.tiles_m;
  const int tj = blockIdx.x / a.tiles_m;
  const int n = tj / a.tiles_per_img;
  const int tq = tj - n * a.tiles_per_img;
  const int p0 = a.tw ? 0 : tq * BN;
  const int oh_first = a.tw ? tq / a.tiles_x * (BN / a.tw) : p0 / a.ow;  // first output row and column of the tile
  const int ow_first = a.tw ? tq % a.tiles_x * a.tw : 0;
  const int i0 = tm * BM;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int RS = a.r * a.s;
  const int K = a.c * RS;
  const int plane = a.nr * a.wp;

  // tap table: offset of tap kk = (c_l, r, s) inside the halo tile; padding taps point at 0 (their
  // kernel-matrix entries are zero).
  for (int kk = tid; kk < a.kch; kk += kThreads) {
    int off = 0;
    if (kk < a.cc * RS) {
      const int cl = kk / RS;
      const int q = kk - cl * RS;
      const int r = q / a.s;
      off = cl * plane + r * a.wp + (q - r * a.s);
    }
    tapoff[kk] = off;
  }

  // this lane's pixels (one per 32-wide accumulator column block)
  int lane_base[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) (void)tile_pixel(a, p0, oh_first, ow_first, wn0 + ni * 32 + l32, &lane_base[ni]);

  SA sa;
  sa.init(tid);
  int64_t a_off[SA::SLOTS];
  bool a_row_ok[SA::SLOTS];
#pragma unroll
  for (int e = 0; e < SA::SLOTS; ++e) {
    const int i = i0 + sa.line(e);
    a_row_ok[e] = i < a.m;
    a_off[e] = (int64_t)(a_row_ok[e] ? i : 0) * K;
  }

  f32x16 acc[TM][TN];
  zero_acc<TM, TN>(acc);

  const T* xin = static_cast<const T*>(a.x) + (int64_t)n * a.c * a.h * a.w;
  const T* wgt = static_cast<const T*>(a.wgt);
  T* yout = static_cast<T*>(a.y);
  const int slabs = a.kch / BK;

  for (int c0 = 0; c0 < a.c; c0 += a.cc) {
    const int cc = min(a.cc, a.c - c0);
    const int kbase = c0 * RS;      // first column of the kernel matrix in this chunk
    const int klen = cc * RS;       // valid taps in this chunk
    // kernel-matrix slab fetch: columns kbase + s*BK + [0, BK), zero beyond klen
    auto fetch = [&](int sl) {
#pragma unroll
      for (int e = 0; e < SA::SLOTS; ++e) {
        const int kk = sl * BK + sa.c;
        sa.ok[e] = a_row_ok[e] && kk < klen;
        const T* src = wgt + a_off[e] + kbase + min(kk, klen - (VEC ? 4 : 1));
        if (VEC) {
          const float4 t = ld4(src);
          sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
        } else {
          sa.v[e][0] = ld(src);
        }
      }
    };
    fetch(0);
    __syncthreads();  // previous chunk's MFMAs are done with the halo tile and the A slabs
    // stage the halo rows of this chunk: input rows oh_first - ph + [0, nr), columns -pw + [0, wp)
    stage_halo<8>(halo, xin + (int64_t)c0 * a.h * a.w, cc, cc, a.nr, a.wp, a.h, a.w, oh_first - a.ph, a.pw - ow_first, tid);
    sa.store(As0);
    __syncthreads();

    for (int sl = 0; sl < slabs; ++sl) {
      const int cur = sl & 1;
      if (sl * BK >= klen) break;  // a short last chunk needs fewer slabs (uniform across the block)
      const bool more = (sl + 1) * BK < klen;
      if (more) fetch(sl + 1);
      const float* As = As0 + cur * LA::SIZE;
      const int* toff = tapoff + sl * BK;
#pragma unroll
      for (int t = 0; t < BK / 8; ++t) {
        float4 af[TM];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi) af[mi] = load_frag<BM, BK, true>(As, wm0 + mi * 32, t, lane);
        const int4 o4 = *reinterpret_cast<const int4*>(toff + 8 * t + 4 * half);
        const int o[4] = {o4.x, o4.y, o4.z, o4.w};
        float bf[TN][4];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
          for (int i = 0; i < 4; ++i) bf[ni][i] = halo[lane_base[ni] + o[i]];
        const float* afl = reinterpret_cast<const float*>(af);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(afl[mi * 4 + i], bf[ni][i], acc[mi][ni], 0, 0, 0);
      }
      if (more) sa.store(As0 + (cur ^ 1) * LA::SIZE);
      __syncthreads();
    }
  }

#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    int unused;
    const int p = tile_pixel(a, p0, oh_first, ow_first, wn0 + ni * 32 + l32, &unused);
    if (p < 0) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row(q, lane);
        if (i < a.m) {
          float v = acc[mi][ni][q];
          if (a.bias) v += a.bias[i];
          if (a.relu) v = fmaxf(v, 0.f);
          st(yout + ((int64_t)n * a.m + i) * a.P + p, v);
        }
      }
  }
}

// The same kernel for 33..48 output maps (BM = 48), on the 16 x 16 x 4 form of the instruction: 32-row tiles
// would run such a layer as 64 rows, a quarter of them padding.  Every wave holds all 48 rows (three 16-row
// tiles) for WN of the block's pixels.  Lane l feeds row / pixel l % 16 and, of a group of 16 contraction
// indices, the four 4*(l / 16) + [0, 4): step i of the group contracts index 4*(l / 16) + i on every lane,
// the kernel-matrix slab and the tap table being read with the same permutation.
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int BM, int BN, int WN, int BK, bool VEC, typename T>
__global__ __launch_bounds__(kThreads) void conv_halo16_kernel(HaloArgs a) {
  static_assert((BN / WN) * 64 == kThreads, "four waves per block, side by side along the pixels");
  static_assert(BM % 16 == 0 && WN % 16 == 0 && BK % 16 == 0, "16-wide tiles");
  using LA = LdsTile<BM, BK, true>;
  using SA = Stager<BM, BK, kThreads, true, VEC>;
  constexpr int TM = BM / 16, TN = WN / 16;
  extern __shared__ float4 smem4[];
  float* const As0 = reinterpret_cast<float*>(smem4);              // 2 slabs of the kernel matrix
  int* const tapoff = reinterpret_cast<int*>(As0 + 2 * LA::SIZE);  // [kch]
  float* const halo = As0 + 2 * LA::SIZE + a.kch;                  // [cc][nr][wp]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;
  const int tm = blockIdx.x % a.tiles_m;
  const int tj = blockIdx.x / a.tiles_m;
  const int n = tj / a.tiles_per_img;
  const int tq = tj - n * a.tiles_per_img;
  const int p0 = a.tw ? 0 : tq * BN;
  const int oh_first = a.tw ? tq / a.tiles_x * (BN / a.tw) : p0 / a.ow;  // first output row and column of the tile
  const int ow_first = a.tw ? tq % a.tiles_x * a.tw : 0;
  const int i0 = tm * BM;
  const int wn0 = wave * WN;
  const int RS = a.r * a.s;
  const int K = a.c * RS;
  const int plane = a.nr * a.wp;

  for (int kk = tid; kk < a.kch; kk += kThreads) {  // tap table, as above
    int off = 0;
    if (kk < a.cc * RS) {
      const int cl = kk / RS;
      const int q = kk - cl * RS;
      const int r = q / a.s;
      off = cl * plane + r * a.wp + (q - r * a.s);
    }
    tapoff[kk] = off;
  }

  int lane_base[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) (void)tile_pixel(a, p0, oh_first, ow_first, wn0 + ni * 16 + l16, &lane_base[ni]);

  SA sa;
  sa.init(tid);
  int64_t a_off[SA::SLOTS];
  bool a_row_ok[SA::SLOTS];
#pragma unroll
  for (int e = 0; e < SA::SLOTS; ++e) {
    const int i = i0 + sa.line(e);
    a_row_ok[e] = i < a.m && sa.line(e) < BM;
    a_off[e] = (int64_t)(a_row_ok[e] ? i : 0) * K;
  }

  f32x4 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[mi][ni][q] = 0.f;

  const T* xin = static_cast<const T*>(a.x) + (int64_t)n * a.c * a.h * a.w;
  const T* wgt = static_cast<const T*>(a.wgt);
  T* yout = static_cast<T*>(a.y);
  const int slabs = a.kch / BK;

  for (int c0 = 0; c0 < a.c; c0 += a.cc) {
    const int cc = min(a.cc, a.c - c0);
    const int kbase = c0 * RS;
    const int klen = cc * RS;
    auto fetch = [&](int sl) {
#pragma unroll
      for (int e = 0; e < SA::SLOTS; ++e) {
        const int kk = sl * BK + sa.c;
        sa.ok[e] = a_row_ok[e] && kk < klen;
        const T* src = wgt + a_off[e] + kbase + min(kk, klen - (VEC ? 4 : 1));
        if (VEC) {
          const float4 t = ld4(src);
          sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
        } else {
          sa.v[e][0] = ld(src);
        }
      }
    };
    fetch(0);
    __syncthreads();  // previous chunk's MFMAs are done with the halo tile and the A slabs
    stage_halo<8>(halo, xin + (int64_t)c0 * a.h * a.w, cc, cc, a.nr, a.wp, a.h, a.w, oh_first - a.ph, a.pw - ow_first, tid);
    sa.store(As0);
    __syncthreads();

    for (int sl = 0; sl < slabs; ++sl) {
      const int cur = sl & 1;
      if (sl * BK >= klen) break;
      const bool more = (sl + 1) * BK < klen;
      if (more) fetch(sl + 1);
      const float* As = As0 + cur * LA::SIZE;
      const int* toff = tapoff + sl * BK;
#pragma unroll
      for (int t = 0; t < BK / 16; ++t) {
        float4 af[TM];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
          af[mi] = *reinterpret_cast<const float4*>(As + (mi * 16 + l16) * LA::PITCH + 16 * t + 4 * kq);
        const int4 o4 = *reinterpret_cast<const int4*>(toff + 16 * t + 4 * kq);
        const int o[4] = {o4.x, o4.y, o4.z, o4.w};
        float bf[TN][4];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
          for (int i = 0; i < 4; ++i) bf[ni][i] = halo[lane_base[ni] + o[i]];
        const float* afl = reinterpret_cast<const float*>(af);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x4f32(afl[mi * 4 + i], bf[ni][i], acc[mi][ni], 0, 0, 0);
      }
      if (more) sa.store(As0 + (cur ^ 1) * LA::SIZE);
      __syncthreads();
    }
  }

  // 16 x 16 result: register q of lane l holds row 4*(l / 16) + q, column l % 16
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    int unused;
    const int p = tile_pixel(a, p0, oh_first, ow_first, wn0 + ni * 16 + l16, &unused);
    if (p < 0) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = i0 + mi * 16 + 4 * kq + q;
        if (i < a.m) {
          float v = acc[mi][ni][q];
          if (a.bias) v += a.bias[i];
          if (a.relu) v = fmaxf(v, 0.f);
          st(yout + ((int64_t)n * a.m + i) * a.P + p, v);
        }
      }
  }
}

// w2[c][m][r'][s'] = w[m][c][R-1-r'][S-1-s']: the kernel matrix of the input-gradient correlation.
template <typename T>
__global__ __launch_bounds__(kThreads) void flip_transpose_kernel(const T* __restrict__ w, T* __restrict__ w2, int M,
                                                                  int C, int RS) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= (int64_t)M * C * RS) return;
  const int q = (int)(i % RS);
  const int64_t t = i / RS;
  const int m = (int)(t % M);
  const int c = (int)(t / M);
  w2[i] = w[((int64_t)m * C + c) * RS + (RS - 1 - q)];
}

vcnn_status launch_flip_transpose(int dtype, const void* w, void* w2, int M, int C, int RS, hipStream_t st) {
  const int64_t count = (int64_t)M * C * RS;
  const dim3 grid((unsigned)ceil_div(count, kThreads)), block(kThreads);
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL(flip_transpose_kernel<bf16>, grid, block, 0, st, (const bf16*)w, (bf16*)w2, M, C, RS);
  else
    hipLaunchKernelGGL(flip_transpose_kernel<float>, grid, block, 0, st, (const float*)w, (float*)w2, M, C, RS);
  return check_launch("flip_transpose");
}

// ---- planning -------------------------------------------------------------------------------------------
static constexpr size_t kLdsBudget = 76 * 1024;  // two blocks per CU out of 160 KB
// 128-row tiles (64 accumulator + about 75 other registers per lane) fit three waves per SIMD and measure
// faster with three smaller blocks per CU than with two (cfg5 c3 forward 3.29 -> 3.17 ms); the narrower tiles
// stage their halo tile more often with a smaller budget and lose more than they gain.
static constexpr size_t kLdsBudget3 = 52 * 1024;

static int halo_bm(int m) { return m <= 32 ? 32 : (m <= 48 ? 48 : (m <= 64 ? 64 : 128)); }
// Pixel tile: the widest tile unless a narrower one pads a small image less.  Narrow tiles do fewer MFMAs
// per LDS read, so they carry a handicap - but only once the launch fills the chip; below that, more and
// shorter blocks win.
static int halo_bn(int m, int64_t P, int n) {
  const int widest = m <= 32 ? 512 : (m <= 64 ? 256 : 128);
  const int64_t row_tiles = ceil_div(m, halo_bm(m));
  int best = 0;
  double best_cost = 0;
  for (int bn = widest; bn >= 64; bn /= 2) {
    if (m <= 32 && bn < 128) break;  // 32-row tiles keep their four waves side by side
    const int64_t tiles = row_tiles * n * ceil_div(P, bn);
    // the handicap applies once the next wider tile already fills the chip (512 resident blocks): narrowing a launch
    // that leaves compute units idle, or with one block each, costs nothing
    const int64_t wider_tiles = bn == widest ? tiles : row_tiles * n * ceil_div(P, 2 * bn);
    const double handicap = wider_tiles >= 512 ? (bn == widest ? 1.0 : (2 * bn == widest ? 1.1 : 1.25)) : 1.0;
    const double cost = (double)ceil_div(P, bn) * bn * handicap;
    if (best == 0 || cost < best_cost - 1e-9 || (cost < best_cost + 1e-9 && tiles <= 1024)) best = bn, best_cost = cost;
  }
  return best;
}
// Slab depth: narrow row tiles do few MFMAs per slab, so they take deeper slabs (fewer barriers per MFMA).
static int halo_bk(int m, int64_t K) {
  if (m <= 64 && m > 48 && K <= 128 && ceil_div(K, 32) * 32 < ceil_div(K, 64) * 64) return 32;  // a short contraction pads less
  return m <= 64 ? 64 : 32;
}

// Strip width for tiles of bn pixels: the widest of 32, 16, 8 columns unless a narrower strip pads the plane clearly less
// (narrow strips store short row segments).
static int strip_width(int bn, int oh, int ow) {
  int best = 0;
  double best_cost = 0;
  for (int tw = 32; tw >= 8; tw /= 2) {
    const int th = bn / tw;
    const double cost = (double)ceil_div(oh, th) * th * ceil_div(ow, tw) * tw * (tw == 32 ? 1.0 : (tw == 16 ? 1.1 : 1.3));
    if (best == 0 || cost < best_cost) best = tw, best_cost = cost;
  }
  return best;
}

bool conv_halo_plan(int n, int c, int h, int w, int m, int r, int s, int ph, int pw, HaloPlan* p) {
  const int oh = h + 2 * ph - r + 1, ow = w + 2 * pw - s + 1;
  if (oh <= 0 || ow <= 0 || (int64_t)c * h * w > 0x7fffffffLL) return false;  // 32-bit offsets inside a sample
  const int bm = halo_bm(m), bn = halo_bn(m, (int64_t)oh * ow, n);
  int BK = halo_bk(m, (int64_t)c * r * s);
  if (bm == 64 && bn != 256) BK = 64;  // the 32-deep variant exists for the widest pixel tile only
  const int rs = r * s;
  const size_t a_bytes = 2 * (size_t)(BK + 4) * bm * sizeof(float);
  // largest channel chunk that fits the LDS budget with a tap table of at most 2048 entries
  auto largest_chunk = [&](int nr, int wp) {
    int best = 0;
    for (int cc = 1; cc <= c; ++cc) {
      const int kch = (int)ceil_div((int64_t)cc * rs, BK) * BK;
      const size_t bytes = a_bytes + (size_t)kch * 4 + (size_t)cc * nr * wp * 4;
      if (bytes > (bm == 128 ? kLdsBudget3 : kLdsBudget) || kch > 2048) break;
      best = cc;
    }
    return best;
  };
  // Tiles are runs of bn consecutive pixels (whole rows of the plane in the halo tile).  A tall kernel on a wide plane
  // makes that tile too large for even one channel (121 x 1 taps on 184 columns: 123 rows x 184); then the tile is a
  // strip of bn / tw rows x tw columns, whose halo is as narrow as the strip.
  int rows = (bn + ow - 2) / ow + 1;  // rows a run of bn consecutive pixels can touch
  if (rows > oh) rows = oh;
  int nr = rows + r - 1, wp = w + 2 * pw, tw = 0;
  int best = largest_chunk(nr, wp);
  if (best == 0) {
    tw = strip_width(bn, oh, ow);
    nr = bn / tw + r - 1, wp = tw + s - 1;
    // one-column kernels: the lane groups of a step read rows 4 apart; a pitch of 4 (16-row tiles: four groups) or
    // 8 (32-row tiles: two groups) modulo 16 puts them on different banks
    if (s == 1) wp += ((bm == 48 ? 4 : 8) - wp % 16 + 16) % 16;
    best = largest_chunk(nr, wp);
    if (best == 0) return false;
  }
  // prefer a chunk whose tap count fills its last slab (fewest zero taps), among chunks at least half as large
  int pick = best;
  double pick_waste = 2.0;
  const bool k_vec = ((int64_t)c * rs) % 4 == 0;
  bool any_vec = false;
  for (int cc = best; cc >= 1 && 2 * cc > best; --cc) any_vec |= k_vec && ((int64_t)cc * rs) % 4 == 0;
  for (int cc = best; cc >= 1 && 2 * cc > best; --cc) {
    if (any_vec && ((int64_t)cc * rs) % 4 != 0) continue;  // keep 16-byte kernel-matrix loads when possible
    const int64_t chunks = ceil_div(c, cc);
    // slabs actually executed: full chunks use ceil(cc*rs/BK); the last may be shorter
    const int last = c - (int)(chunks - 1) * cc;
    const int64_t slabs = (chunks - 1) * ceil_div((int64_t)cc * rs, BK) + ceil_div((int64_t)last * rs, BK);
    const double waste = 1.0 - (double)c * rs / (double)(slabs * BK);
    if (waste < pick_waste - 1e-9) pick = cc, pick_waste = waste;
  }
  p->bm = bm, p->bn = bn, p->bk = BK, p->cc = pick, p->nr = nr, p->wp = wp, p->tw = tw;
  p->kch = (int)ceil_div((int64_t)pick * rs, BK) * BK;
  p->lds_bytes = a_bytes + (size_t)p->kch * 4 + (size_t)pick * nr * wp * 4;
  p->vec = ((int64_t)c * rs) % 4 == 0 && ((int64_t)pick * rs) % 4 == 0;
  p->tiles_per_img = tw ? ceil_div(oh, bn / tw) * ceil_div(ow, tw) : ceil_div((int64_t)oh * ow, bn);
  const int64_t tiles = ceil_div(m, bm) * (int64_t)n * p->tiles_per_img;
  return tiles <= 0x7fffffffLL;
}

template <int BM, int BN, int WM, int WN, int BK, bool VEC, typename T>
static void launch_halo_one(const HaloArgs& a, const HaloPlan& p, hipStream_t st) {
  const dim3 grid((unsigned)((int64_t)a.tiles_m * a.n * a.tiles_per_img)), block(kThreads);
  auto kernel = conv_halo_kernel<BM, BN, WM, WN, BK, VEC, T>;
  static bool opted = false;  // one flag per instantiation, i.e. per kernel
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsBudget);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, st, a);
}

template <int BM, int BN, int WM, int WN, int BK>
static void launch_halo(const HaloArgs& a, const HaloPlan& p, bool vec, int dtype, hipStream_t st) {
  if (dtype == VCNN_BF16) {
    if (vec) launch_halo_one<BM, BN, WM, WN, BK, true, bf16>(a, p, st);
    else launch_halo_one<BM, BN, WM, WN, BK, false, bf16>(a, p, st);
  } else {
    if (vec) launch_halo_one<BM, BN, WM, WN, BK, true, float>(a, p, st);
    else launch_halo_one<BM, BN, WM, WN, BK, false, float>(a, p, st);
  }
}

template <int BN, bool VEC, typename T>
static void launch_halo16_one(const HaloArgs& a, const HaloPlan& p, hipStream_t st) {
  const dim3 grid((unsigned)((int64_t)a.tiles_m * a.n * a.tiles_per_img)), block(kThreads);
  auto kernel = conv_halo16_kernel<48, BN, BN / 4, 64, VEC, T>;
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsBudget);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, st, a);
}

// 48-row tiles: pixel tiles of 256, 128 or 64
static void launch_halo16(const HaloArgs& a, const HaloPlan& p, bool vec, int dtype, hipStream_t st) {
  auto go = [&](auto bn_tag) {
    constexpr int BN = decltype(bn_tag)::value;
    if (dtype == VCNN_BF16) {
      if (vec) launch_halo16_one<BN, true, bf16>(a, p, st);
      else launch_halo16_one<BN, false, bf16>(a, p, st);
    } else {
      if (vec) launch_halo16_one<BN, true, float>(a, p, st);
      else launch_halo16_one<BN, false, float>(a, p, st);
    }
  };
  if (p.bn == 256) go(std::integral_constant<int, 256>{});
  else if (p.bn == 128) go(std::integral_constant<int, 128>{});
  else go(std::integral_constant<int, 64>{});
}

vcnn_status launch_conv_halo(const HaloPlan& p, int dtype, int n, int c, int h, int w, int m, int r, int s, int ph,
                             int pw, const void* x, const void* wgt, const float* bias, void* y, int relu,
                             hipStream_t st) {
  HaloArgs a{};
  a.x = x, a.wgt = wgt, a.bias = bias, a.y = y;
  a.n = n, a.c = c, a.h = h, a.w = w, a.m = m, a.r = r, a.s = s, a.ph = ph, a.pw = pw;
  a.oh = h + 2 * ph - r + 1, a.ow = w + 2 * pw - s + 1;
  a.P = a.oh * a.ow;
  a.tiles_m = (int)ceil_div(m, p.bm);
  a.tiles_per_img = (int)p.tiles_per_img;
  a.tw = p.tw, a.tiles_x = p.tw ? (int)ceil_div(a.ow, p.tw) : 0;
  a.cc = p.cc, a.nr = p.nr, a.wp = p.wp, a.kch = p.kch, a.relu = relu;
  const bool vec = p.vec && (dtype == VCNN_BF16 ? group_aligned<bf16>(wgt) : group_aligned<float>(wgt));
  if (p.bm == 32 && p.bn == 512)
    launch_halo<32, 512, 32, 128, 64>(a, p, vec, dtype, st);
  else if (p.bm == 32 && p.bn == 256)
    launch_halo<32, 256, 32, 64, 64>(a, p, vec, dtype, st);
  else if (p.bm == 32)
    launch_halo<32, 128, 32, 32, 64>(a, p, vec, dtype, st);
  else if (p.bm == 48)
    launch_halo16(a, p, vec, dtype, st);
  else if (p.bm == 64 && p.bn == 256 && p.bk == 32)
    launch_halo<64, 256, 64, 64, 32>(a, p, vec, dtype, st);
  else if (p.bm == 64 && p.bn == 256)
    launch_halo<64, 256, 64, 64, 64>(a, p, vec, dtype, st);
  else if (p.bm == 64 && p.bn == 128)
    launch_halo<64, 128, 32, 64, 64>(a, p, vec, dtype, st);
  else if (p.bm == 64)
    launch_halo<64, 64, 32, 32, 64>(a, p, vec, dtype, st);
  else if (p.bn == 128)
    launch_halo<128, 128, 64, 64, 32>(a, p, vec, dtype, st);
  else
    launch_halo<128, 64, 32, 64, 32>(a, p, vec, dtype, st);
  return check_launch("conv_halo");
}

}  // namespace vcnn

// =========================================================================================================
// Implicit-unroll filter gradient: dW[m][(c,r,s)] = sum_{n,pixel} dY[n][m][pixel] * xpad[n][c][pixel + (r,s)].
// The product dY * phi_c(x)^T without phi_c(x): a block owns BM output maps x BNK columns of the kernel
// matrix (a run of taps, possibly spanning several input channels) and walks over runs of BP output
// pixels.  Per run it stages the input rows (with halo) of the channels it needs in LDS; dY streams
// through double-buffered slabs as the A operand (contraction index = pixel), and the B operand is read
// from the halo tile at tap_base(lane) + pixel_offset(step).  The contraction is split over blocks
// (blockIdx.y); the partial products are added in a fixed order by a second kernel.
// =========================================================================================================
namespace vcnn {

struct HaloFilterArgs {
  const void* x;     // [n][c][h][w]     element type T (float or bf16)
  const void* dy;    // [n][m][oh][ow]   element type T
  float* out;        // [splits][m][Kp]
  int n, c, h, w, m, r, s, ph, pw, oh, ow, P;
  int Kp;            // row pitch of out: c*r*s, or c*r*s + 1 when column c*r*s carries the bias gradient
  int tiles_m;
  int bp;            // pixels per run (multiple of BK)
  int runs_per_img;
  int runs_per_split;
  int ccs;           // channels a block's column range can span
  int nr, wp;
};

template <int BM, int BNK, int WM, int WN, int BK, bool VEC, typename T>
__global__ __launch_bounds__(kThreads) void conv_halo_filter_kernel(HaloFilterArgs a) {
  static_assert((BM / WM) * (BNK / WN) * 64 == kThreads, "four waves per block");
  using LA = LdsTile<BM, BK, true>;
  using SA = Stager<BM, BK, kThreads, true, VEC>;
  constexpr int TM = WM / 32, TN = WN / 32;
  extern __shared__ float4 smem4[];
  float* const As0 = reinterpret_cast<float*>(smem4);
  int* const pixoff = reinterpret_cast<int*>(As0 + 2 * LA::SIZE);  // [bp]
  float* const halo = As0 + 2 * LA::SIZE + a.bp;                   // [ccs][nr][wp]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int tm = blockIdx.x % a.tiles_m;
  const int tk = blockIdx.x / a.tiles_m;
  const int i0 = tm * BM, k0 = tk * BNK;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int RS = a.r * a.s;
  const int K = a.c * RS;
  const int plane = a.nr * a.wp;
  const int c_first = k0 / RS;

  // this lane's kernel-matrix columns: offset of tap (c, r, s) inside the halo tile.  Column K, when the
  // output has room for it, is the bias gradient, the sum over pixels of dY times one: its lane reads a plane
  // of ones kept behind the staged channels (dY is zero beyond a run's last pixel, so the ones need no mask).
  int tap_base[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = min(k0 + wn0 + ni * 32 + l32, K - 1);
    const int c = col / RS;
    const int q = col - c * RS;
    const int r = q / a.s;
    tap_base[ni] = (c - c_first) * plane + r * a.wp + (q - r * a.s);
    if (a.Kp > K && k0 + wn0 + ni * 32 + l32 == K) tap_base[ni] = a.ccs * plane;
  }
  if (a.Kp > K)
    for (int e = tid; e < plane; e += kThreads) halo[a.ccs * plane + e] = 1.f;  // published by the first run's barrier

  SA sa;
  sa.init(tid);
  const bool wave_has_columns = k0 + wn0 < a.Kp;

  f32x16 acc[TM][TN];
  zero_acc<TM, TN>(acc);

  const int total_runs = a.n * a.runs_per_img;
  const int run0 = blockIdx.y * a.runs_per_split;
  const int run1 = min(total_runs, run0 + a.runs_per_split);
  const int slabs_per_run = a.bp / BK;

  for (int run = run0; run < run1; ++run) {
    const int n = run / a.runs_per_img;
    const int p0 = (run - n * a.runs_per_img) * a.bp;
    const int plen = min(a.bp, a.P - p0);  // valid pixels in this run
    const int oh_first = p0 / a.ow;
    const T* dyn = static_cast<const T*>(a.dy) + (int64_t)n * a.m * a.P + p0;
    auto fetch = [&](int sl) {
      const int pk = sl * BK + sa.c;  // pixel inside the run
#pragma unroll
      for (int e = 0; e < SA::SLOTS; ++e) {
        const int m = i0 + sa.line(e);
        sa.ok[e] = m < a.m && pk < plen;
        const T* src = dyn + (int64_t)min(m, a.m - 1) * a.P + min(pk, plen - (VEC ? 4 : 1));
        if constexpr (VEC && std::is_same<T, float>::value) {
          // rows of dY start at any dword (odd pixel counts): a 16-byte load at dword alignment.  A run's last group
          // of four may end before its fourth pixel: the load is moved back to the last four pixels (plen >= 4 by
          // the plan) and the wanted ones are shifted down, zeros behind them.
          const float4 t = ld4_dword_aligned(src);
          const int d = pk - min(pk, plen - 4);
          sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
          if (d > 0 && d < 4) {
            sa.v[e][0] = d == 1 ? t.y : (d == 2 ? t.z : t.w);
            sa.v[e][1] = d == 1 ? t.z : (d == 2 ? t.w : 0.f);
            sa.v[e][2] = d == 1 ? t.w : 0.f;
            sa.v[e][3] = 0.f;
          }
        } else if constexpr (VEC) {
          const float4 t = ld4(src);
          sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
        } else {
          sa.v[e][0] = ld(src);
        }
      }
    };
    fetch(0);
    __syncthreads();  // the previous run's MFMAs are done with the halo tile, the table and the slabs
    for (int pk = tid; pk < a.bp; pk += kThreads) {
      const int p = min(p0 + pk, a.P - 1);
      const int oh = p / a.ow;
      pixoff[pk] = (oh - oh_first) * a.wp + (p - oh * a.ow);
    }
    stage_halo<8>(halo, static_cast<const T*>(a.x) + ((int64_t)n * a.c + c_first) * a.h * a.w, a.ccs, a.c - c_first,
                  a.nr, a.wp, a.h, a.w, oh_first - a.ph, a.pw, tid);
    sa.store(As0);
    __syncthreads();

    for (int sl = 0; sl < slabs_per_run; ++sl) {
      const int cur = sl & 1;
      if (sl * BK >= plen) break;
      const bool more = (sl + 1) * BK < plen;
      if (more) fetch(sl + 1);
      const float* As = As0 + cur * LA::SIZE;
      const int* poff = pixoff + sl * BK;
      // (a wave whose columns all lie beyond the matrix - the last column tile of a matrix that fills a fraction of
      // it - stages and synchronises with the others but multiplies nothing)
      if (wave_has_columns)
#pragma unroll
      for (int t = 0; t < BK / 8; ++t) {
        float4 af[TM];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi) af[mi] = load_frag<BM, BK, true>(As, wm0 + mi * 32, t, lane);
        const int4 o4 = *reinterpret_cast<const int4*>(poff + 8 * t + 4 * half);
        const int o[4] = {o4.x, o4.y, o4.z, o4.w};
        float bf[TN][4];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
          for (int i = 0; i < 4; ++i) bf[ni][i] = halo[tap_base[ni] + o[i]];
        const float* afl = reinterpret_cast<const float*>(af);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(afl[mi * 4 + i], bf[ni][i], acc[mi][ni], 0, 0, 0);
      }
      if (more) sa.store(As0 + (cur ^ 1) * LA::SIZE);
      __syncthreads();
    }
  }

  float* dst = a.out + (int64_t)blockIdx.y * a.m * a.Kp;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = k0 + wn0 + ni * 32 + l32;
    if (col >= a.Kp) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int m = i0 + wm0 + mi * 32 + acc_row(q, lane);
        if (m < a.m) dst[(int64_t)m * a.Kp + col] = acc[mi][ni][q];
      }
  }
}

// The same kernel for 33..48 output maps (BM = 48) on the 16 x 16 x 4 form of the instruction (as the forward kernel
// above: 32-row tiles would run such a layer as 64 rows, a quarter of them padding).  Every wave holds all 48 rows
// for WN of the block's kernel-matrix columns.  Lane l feeds row / column l % 16 and, of a group of 16 pixels, the
// four 4*(l / 16) + [0, 4); the dY slab and the pixel-offset table are read with the same permutation.
template <int BM, int BNK, int WN, int BK, bool VEC, typename T>
__global__ __launch_bounds__(kThreads) void conv_halo_filter16_kernel(HaloFilterArgs a) {
  static_assert((BNK / WN) * 64 == kThreads, "four waves per block, side by side along the columns");
  static_assert(BM % 16 == 0 && WN % 16 == 0 && BK % 16 == 0, "16-wide tiles");
  using LA = LdsTile<BM, BK, true>;
  using SA = Stager<BM, BK, kThreads, true, VEC>;
  constexpr int TM = BM / 16, TN = WN / 16;
  extern __shared__ float4 smem4[];
  float* const As0 = reinterpret_cast<float*>(smem4);
  int* const pixoff = reinterpret_cast<int*>(As0 + 2 * LA::SIZE);  // [bp]
  float* const halo = As0 + 2 * LA::SIZE + a.bp;                   // [ccs][nr][wp]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;
  const int tm = blockIdx.x % a.tiles_m;
  const int tk = blockIdx.x / a.tiles_m;
  const int i0 = tm * BM, k0 = tk * BNK;
  const int wn0 = wave * WN;
  const int RS = a.r * a.s;
  const int K = a.c * RS;
  const int plane = a.nr * a.wp;
  const int c_first = k0 / RS;

  int tap_base[TN];  // as above; column K, when there is room for it, reads the plane of ones (bias gradient)
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = min(k0 + wn0 + ni * 16 + l16, K - 1);
    const int c = col / RS;
    const int q = col - c * RS;
    const int r = q / a.s;
    tap_base[ni] = (c - c_first) * plane + r * a.wp + (q - r * a.s);
    if (a.Kp > K && k0 + wn0 + ni * 16 + l16 == K) tap_base[ni] = a.ccs * plane;
  }
  if (a.Kp > K)
    for (int e = tid; e < plane; e += kThreads) halo[a.ccs * plane + e] = 1.f;  // published by the first run's barrier

  SA sa;
  sa.init(tid);

  f32x4 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[mi][ni][q] = 0.f;

  const int total_runs = a.n * a.runs_per_img;
  const int run0 = blockIdx.y * a.runs_per_split;
  const int run1 = min(total_runs, run0 + a.runs_per_split);
  const int slabs_per_run = a.bp / BK;

  for (int run = run0; run < run1; ++run) {
    const int n = run / a.runs_per_img;
    const int p0 = (run - n * a.runs_per_img) * a.bp;
    const int plen = min(a.bp, a.P - p0);
    const int oh_first = p0 / a.ow;
    const T* dyn = static_cast<const T*>(a.dy) + (int64_t)n * a.m * a.P + p0;
    auto fetch = [&](int sl) {
      const int pk = sl * BK + sa.c;
#pragma unroll
      for (int e = 0; e < SA::SLOTS; ++e) {
        const int m = i0 + sa.line(e);
        sa.ok[e] = m < a.m && pk < plen;
        const T* src = dyn + (int64_t)min(m, a.m - 1) * a.P + min(pk, plen - (VEC ? 4 : 1));
        if constexpr (VEC && std::is_same<T, float>::value) {
          const float4 t = ld4_dword_aligned(src);  // as above: the run's last group is moved back and shifted down
          const int d = pk - min(pk, plen - 4);
          sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
          if (d > 0 && d < 4) {
            sa.v[e][0] = d == 1 ? t.y : (d == 2 ? t.z : t.w);
            sa.v[e][1] = d == 1 ? t.z : (d == 2 ? t.w : 0.f);
            sa.v[e][2] = d == 1 ? t.w : 0.f;
            sa.v[e][3] = 0.f;
          }
        } else if constexpr (VEC) {
          const float4 t = ld4(src);
          sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
        } else {
          sa.v[e][0] = ld(src);
        }
      }
    };
    fetch(0);
    __syncthreads();  // the previous run's MFMAs are done with the halo tile, the table and the slabs
    for (int pk = tid; pk < a.bp; pk += kThreads) {
      const int p = min(p0 + pk, a.P - 1);
      const int oh = p / a.ow;
      pixoff[pk] = (oh - oh_first) * a.wp + (p - oh * a.ow);
    }
    stage_halo<8>(halo, static_cast<const T*>(a.x) + ((int64_t)n * a.c + c_first) * a.h * a.w, a.ccs, a.c - c_first,
                  a.nr, a.wp, a.h, a.w, oh_first - a.ph, a.pw, tid);
    sa.store(As0);
    __syncthreads();

    for (int sl = 0; sl < slabs_per_run; ++sl) {
      const int cur = sl & 1;
      if (sl * BK >= plen) break;
      const bool more = (sl + 1) * BK < plen;
      if (more) fetch(sl + 1);
      const float* As = As0 + cur * LA::SIZE;
      const int* poff = pixoff + sl * BK;
#pragma unroll
      for (int t = 0; t < BK / 16; ++t) {
        float4 af[TM];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
          af[mi] = *reinterpret_cast<const float4*>(As + (mi * 16 + l16) * LA::PITCH + 16 * t + 4 * kq);
        const int4 o4 = *reinterpret_cast<const int4*>(poff + 16 * t + 4 * kq);
        const int o[4] = {o4.x, o4.y, o4.z, o4.w};
        float bf[TN][4];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
          for (int i = 0; i < 4; ++i) bf[ni][i] = halo[tap_base[ni] + o[i]];
        const float* afl = reinterpret_cast<const float*>(af);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x4f32(afl[mi * 4 + i], bf[ni][i], acc[mi][ni], 0, 0, 0);
      }
      if (more) sa.store(As0 + (cur ^ 1) * LA::SIZE);
      __syncthreads();
    }
  }

  // 16 x 16 result: register q of lane l holds row 4*(l / 16) + q, column l % 16
  float* dst = a.out + (int64_t)blockIdx.y * a.m * a.Kp;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = k0 + wn0 + ni * 16 + l16;
    if (col >= a.Kp) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int m = i0 + mi * 16 + 4 * kq + q;
        if (m < a.m) dst[(int64_t)m * a.Kp + col] = acc[mi][ni][q];
      }
  }
}

// Slab depth (pixels of dY staged per barrier): a narrow row tile does few MFMAs per pixel, so it takes deeper
// slabs - the next slab's loads then have a few microseconds of MFMA work to hide behind.
static int filter_bk(int64_t m) { return m <= 32 ? 128 : (m <= 64 ? 64 : 32); }

bool conv_halo_filter_plan(const ConvGeom& g, HaloFilterPlan* p) {
  const int rs = g.r * g.s;
  const int BK = filter_bk(g.M);
  if ((int64_t)g.c * g.h * g.w > 0x7fffffffLL) return false;  // 32-bit offsets inside a sample
  p->bm = g.M <= 32 ? 32 : (g.M <= 48 ? 48 : (g.M <= 64 ? 64 : 128));
  p->bnk = g.M <= 64 ? 256 : 128;
  p->wp = g.w + 2 * g.pw;
  // channels a run of bnk consecutive kernel-matrix columns can touch
  p->ccs = (int)std::min<int64_t>(g.c, (p->bnk + rs - 2) / rs + 1);
  const size_t a_bytes = 2 * (size_t)(BK + 4) * p->bm * sizeof(float);
  // longest pixel run (multiple of BK, at most 1024 and at most one sample) whose halo fits the budget
  int best = 0;
  for (int bp = BK; bp <= 1024; bp += BK) {
    int rows = (bp + g.ow - 2) / g.ow + 1;
    if (rows > g.oh) rows = g.oh;
    const int nr = rows + g.r - 1;
    const size_t bytes = a_bytes + (size_t)bp * 4 + (size_t)p->ccs * nr * p->wp * 4;
    if (bytes > (p->bm >= 48 ? kLdsBudget3 : kLdsBudget)) break;
    best = bp;
    if (bp >= g.P) break;
  }
  if (best == 0) return false;
  p->bp = best;
  int rows = (best + g.ow - 2) / g.ow + 1;
  if (rows > g.oh) rows = g.oh;
  p->nr = rows + g.r - 1;
  p->lds_bytes = a_bytes + (size_t)best * 4 + (size_t)p->ccs * p->nr * p->wp * 4;
  p->runs_per_img = (int)ceil_div(g.P, best);
  const int64_t tiles = ceil_div(g.M, p->bm) * ceil_div(g.K, p->bnk);
  const int64_t total_runs = (int64_t)g.n * p->runs_per_img;
  // contraction slices: at least enough for about 1024 blocks; among up to twice as many, the count whose blocks
  // fill whole rounds of the resident set best (long blocks: a last round that is half empty costs half a round)
  int64_t want = ceil_div(1024, tiles);
  if (want <= 8) {  // (many slices mean short blocks, whose rounds do not matter - and more partial sums to add)
    const int64_t slots = 256 * (p->bm >= 48 ? 3 : 2);
    double best_fill = 0;
    int64_t best_want = want;
    for (int64_t w = want; w <= 2 * want; ++w) {
      const int64_t per = ceil_div(total_runs, std::min<int64_t>(w, total_runs));
      const int64_t blocks = tiles * ceil_div(total_runs, per);
      const double fill = (double)blocks / (double)(ceil_div(blocks, slots) * slots);
      if (fill > best_fill + 0.02) best_fill = fill, best_want = w;
    }
    want = best_want;
  }
  if (want > total_runs) want = total_runs;
  if (want < 1) want = 1;
  p->runs_per_split = (int)ceil_div(total_runs, want);
  p->splits = (int)ceil_div(total_runs, p->runs_per_split);
  // a spare column in the last column tile takes the bias gradient along; its partials then have K + 1 columns and
  // are split into dW and db by the slice sum even when there is a single slice
  p->bias_column = g.K % p->bnk != 0;
  if (p->bias_column) {  // room for the plane of ones, if the budget still holds
    const size_t with_ones = p->lds_bytes + (size_t)p->nr * p->wp * 4;
    if (with_ones <= kLdsBudget) p->lds_bytes = with_ones;
    else p->bias_column = false;
  }
  p->partial_bytes = p->bias_column ? (size_t)p->splits * g.M * (g.K + 1) * sizeof(float)
                                    : (p->splits > 1 ? (size_t)p->splits * g.M * g.K * sizeof(float) : 0);
  // 16-byte loads of dY: when the pixel count is a multiple of 4 (rows then keep the tensor's alignment); float rows
  // may also start at any dword, as long as every run holds at least four pixels (vec4_any)
  p->vec = g.P % 4 == 0;
  p->vec4_any = g.P >= 4 && (g.P % best == 0 || g.P % best >= 4);
  return tiles <= 0x7fffffffLL && p->splits <= 65535;
}

template <int BM, int BNK, int WM, int WN, int BK, bool VEC, typename T>
static void launch_halo_filter_one(const HaloFilterArgs& a, const HaloFilterPlan& p, int tiles, hipStream_t st) {
  const dim3 grid((unsigned)tiles, (unsigned)p.splits), block(kThreads);
  auto kernel = conv_halo_filter_kernel<BM, BNK, WM, WN, BK, VEC, T>;
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsBudget);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, st, a);
}

template <int BM, int BNK, int WM, int WN, int BK>
static void launch_halo_filter(const HaloFilterArgs& a, const HaloFilterPlan& p, bool vec, int dtype, int tiles,
                               hipStream_t st) {
  if (dtype == VCNN_BF16) {
    if (vec) launch_halo_filter_one<BM, BNK, WM, WN, BK, true, bf16>(a, p, tiles, st);
    else launch_halo_filter_one<BM, BNK, WM, WN, BK, false, bf16>(a, p, tiles, st);
  } else {
    if (vec) launch_halo_filter_one<BM, BNK, WM, WN, BK, true, float>(a, p, tiles, st);
    else launch_halo_filter_one<BM, BNK, WM, WN, BK, false, float>(a, p, tiles, st);
  }
}

template <bool VEC, typename T>
static void launch_halo_filter16_one(const HaloFilterArgs& a, const HaloFilterPlan& p, int tiles, hipStream_t st) {
  const dim3 grid((unsigned)tiles, (unsigned)p.splits), block(kThreads);
  auto kernel = conv_halo_filter16_kernel<48, 256, 64, 64, VEC, T>;
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsBudget);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, st, a);
}

// 48-row tiles (33..48 output maps)
static void launch_halo_filter16(const HaloFilterArgs& a, const HaloFilterPlan& p, bool vec, int dtype, int tiles,
                                 hipStream_t st) {
  if (dtype == VCNN_BF16) {
    if (vec) launch_halo_filter16_one<true, bf16>(a, p, tiles, st);
    else launch_halo_filter16_one<false, bf16>(a, p, tiles, st);
  } else {
    if (vec) launch_halo_filter16_one<true, float>(a, p, tiles, st);
    else launch_halo_filter16_one<false, float>(a, p, tiles, st);
  }
}

vcnn_status launch_conv_halo_filter(const HaloFilterPlan& p, int dtype, const ConvGeom& g, const void* x, const void* dy,
                                    float* dw, float* dbias, float* partial, hipStream_t st) {
  const bool with_bias = p.bias_column && dbias;
  HaloFilterArgs a{};
  a.x = x, a.dy = dy, a.out = (p.splits > 1 || with_bias) ? partial : dw;
  a.Kp = (int)g.K + (with_bias ? 1 : 0);
  a.n = g.n, a.c = g.c, a.h = g.h, a.w = g.w, a.m = g.k, a.r = g.r, a.s = g.s, a.ph = g.ph, a.pw = g.pw;
  a.oh = g.oh, a.ow = g.ow, a.P = (int)g.P;
  a.tiles_m = (int)ceil_div(g.M, p.bm);
  a.bp = p.bp, a.runs_per_img = p.runs_per_img, a.runs_per_split = p.runs_per_split;
  a.ccs = p.ccs, a.nr = p.nr, a.wp = p.wp;
  const int tiles = a.tiles_m * (int)ceil_div(g.K, p.bnk);
  const bool vec = dtype == VCNN_BF16 ? p.vec && group_aligned<bf16>(dy)
                                      : (p.vec && group_aligned<float>(dy)) || (p.vec4_any && (reinterpret_cast<uintptr_t>(dy) & 3) == 0);
  if (p.bm == 48)
    launch_halo_filter16(a, p, vec, dtype, tiles, st);
  else if (p.bm == 32)
    launch_halo_filter<32, 256, 32, 64, 128>(a, p, vec, dtype, tiles, st);
  else if (p.bm == 64)
    launch_halo_filter<64, 256, 64, 64, 64>(a, p, vec, dtype, tiles, st);
  else
    launch_halo_filter<128, 128, 64, 64, 32>(a, p, vec, dtype, tiles, st);
  if (vcnn_status s = check_launch("conv_halo_filter")) return s;
  if (with_bias) return launch_sum_slices_split(partial, dw, dbias, g.M, (int)g.K, p.splits, st);
  if (p.splits == 1) return VCNN_OK;
  return launch_sum_slices(partial, nullptr, dw, VCNN_F32, g.M * g.K, p.splits, 1, 1, 0, st);
}

// =========================================================================================================
// Filter gradient of layers with a narrow kernel matrix (K = C*R*S <= 128 columns, at most 64 maps): the first
// layers of the networks, whose contraction over (sample, pixel) is very long while the result is tiny.
// The kernel above would give such a layer one tile and leave most of its columns and waves idle.  Here
// every block computes the whole M x K result for its share of the pixels: a run of 128 output pixels is
// staged at once (dY rows and the input rows + halo, all loads in flight together), the four waves take
// 32 pixels each, and their partial tiles are added in wave order through LDS.  Blocks write partial
// results that a second kernel adds in a fixed order.
// =========================================================================================================
struct FewColsArgs {
  const void* x;   // [n][c][h][w]
  const void* dy;  // [n][m][oh][ow]
  float* out;      // [blocks][m][Kp]
  int n, c, h, w, m, r, s, ph, pw, oh, ow, P, K;
  int Kp;          // K, or K + 1 when the spare column K carries the bias gradient (B operand = 1 there)
  int runs_per_img, total_runs, runs_per_block;
  int nr, wp;
  int tw, tiles_x;  // tw > 0: a run is a strip of kRunPixels / tw output rows x tw output columns (tiles_x strips side by side)
};

static constexpr int kRunPixels = 128;

template <int TM, int TN, typename T>
__global__ __launch_bounds__(kThreads, 2) void filter_grad_few_cols_kernel(FewColsArgs a) {
  constexpr int BP = kRunPixels, PITCH = BP + 4, ROWS = 32 * TM;
  extern __shared__ float4 smem4[];
  float* const dyt = reinterpret_cast<float*>(smem4);             // [ROWS][PITCH]
  int* const pixoff = reinterpret_cast<int*>(dyt + ROWS * PITCH);  // [BP]
  float* const halo = dyt + ROWS * PITCH + BP;                     // [c][nr][wp]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int RS = a.r * a.s;
  const int plane = a.nr * a.wp;

  int tap_base[TN];
  bool ones[TN];  // this lane's column is the bias column: db[m] = sum over pixels of dY[m][pixel] * 1
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = min(ni * 32 + l32, a.K - 1);
    const int c = col / RS;
    const int q = col - c * RS;
    const int r = q / a.s;
    tap_base[ni] = c * plane + r * a.wp + (q - r * a.s);
    ones[ni] = a.Kp > a.K && ni * 32 + l32 == a.K;
  }

  f32x16 acc[TM][TN];
  zero_acc<TM, TN>(acc);

  const int run0 = blockIdx.x * a.runs_per_block;
  const int run1 = min(a.total_runs, run0 + a.runs_per_block);
  for (int run = run0; run < run1; ++run) {
    const int n = run / a.runs_per_img;
    const int tq = run - n * a.runs_per_img;
    const int p0 = a.tw ? 0 : tq * BP;
    const int oh_first = a.tw ? tq / a.tiles_x * (BP / a.tw) : p0 / a.ow;  // first output row and column of the run
    const int ow_first = a.tw ? tq % a.tiles_x * a.tw : 0;
    __syncthreads();  // the previous run's MFMAs are done with the tiles
    // pixel pk = tid % BP of the run: where it lies in the sample's output plane (-1: outside) and in the halo tile
    constexpr int MSTEP = kThreads / BP;
    const int pk = tid % BP;
    int pix, tile_at;
    if (a.tw) {
      const int ty = pk / a.tw, tx = pk - ty * a.tw;
      const int oh = oh_first + ty, ow = ow_first + tx;
      pix = oh < a.oh && ow < a.ow ? oh * a.ow + ow : -1;
      tile_at = ty * a.wp + tx;
    } else {
      const int p = min(p0 + pk, a.P - 1);
      const int oh = p / a.ow;
      pix = p0 + pk < a.P ? p : -1;
      tile_at = (oh - oh_first) * a.wp + (p - oh * a.ow);
    }
    if (tid < BP) pixoff[tid] = tile_at;
    // dY rows of this run, zero beyond the maps / the sample's pixels.  All of a thread's loads are issued before the
    // halo tile is staged and stored only after it: the run costs one memory round trip, not one per eight loads
    const T* dyn = static_cast<const T*>(a.dy) + (int64_t)n * a.m * a.P + max(pix, 0);
    constexpr int PER = ROWS * BP / kThreads;
    float dyv[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int m = u * MSTEP + tid / BP;
      const bool ok = m < a.m && pix >= 0;
      const float t = ld(dyn + (ok ? (int64_t)m * a.P : 0));
      dyv[u] = ok ? t : 0.f;
    }
    stage_halo<8>(halo, static_cast<const T*>(a.x) + (int64_t)n * a.c * a.h * a.w, a.c, a.c, a.nr, a.wp, a.h, a.w,
                  oh_first - a.ph, a.pw - ow_first, tid);
#pragma unroll
    for (int u = 0; u < PER; ++u) dyt[(u * MSTEP + tid / BP) * PITCH + pk] = dyv[u];
    __syncthreads();

#pragma unroll
    for (int g = 0; g < 4; ++g) {  // this wave's 32 pixels in groups of 8 = four MFMA steps
      const int pk0 = wave * 32 + g * 8 + 4 * half;
      float4 af[TM];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi) af[mi] = *reinterpret_cast<const float4*>(dyt + (mi * 32 + l32) * PITCH + pk0);
      const int4 o4 = *reinterpret_cast<const int4*>(pixoff + pk0);
      const int o[4] = {o4.x, o4.y, o4.z, o4.w};
      float bf[TN][4];
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float t = halo[tap_base[ni] + o[i]];
          bf[ni][i] = ones[ni] ? 1.f : t;
        }
      const float* afl = reinterpret_cast<const float*>(af);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(afl[mi * 4 + i], bf[ni][i], acc[mi][ni], 0, 0, 0);
    }
  }

  // add the four waves' tiles in wave order
  float* red = reinterpret_cast<float*>(smem4);  // [TM*TN*16][64 lanes]
#pragma unroll 1
  for (int k = 1; k < 4; ++k) {
    __syncthreads();
    if (wave == k) {
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
          for (int q = 0; q < 16; ++q) red[((mi * TN + ni) * 16 + q) * 64 + lane] = acc[mi][ni][q];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
          for (int q = 0; q < 16; ++q) acc[mi][ni][q] += red[((mi * TN + ni) * 16 + q) * 64 + lane];
    }
  }
  if (wave != 0) return;
  float* dst = a.out + (int64_t)blockIdx.x * a.m * a.Kp;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = ni * 32 + l32;
    if (col >= a.Kp) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int m = mi * 32 + acc_row(q, lane);
        if (m < a.m) dst[(int64_t)m * a.Kp + col] = acc[mi][ni][q];
      }
  }
}

bool filter_grad_few_cols_plan(const ConvGeom& g, FewColsPlan* p) {
  if (g.K > 128 || g.M > 64 || (int64_t)g.c * g.h * g.w > 0x7fffffffLL || g.P > 0x7fffffffLL) return false;
  p->tm = g.M <= 32 ? 1 : 2;
  p->tn = (int)ceil_div(g.K, 32);
  int rows = (kRunPixels + g.ow - 2) / g.ow + 1;  // rows a run of consecutive pixels can touch
  if (rows > g.oh) rows = g.oh;
  p->nr = rows + g.r - 1, p->wp = g.w + 2 * g.pw, p->tw = 0;
  const size_t tile = (size_t)32 * p->tm * (kRunPixels + 4) * 4;
  p->lds_bytes = tile + kRunPixels * 4 + (size_t)g.c * p->nr * p->wp * 4;
  if (p->lds_bytes > 64 * 1024) {
    // a tall kernel on a wide plane: runs are strips of rows x columns, whose halo tile is as narrow as the strip
    // (one-column kernels: an odd pitch keeps the lanes of a step, which read consecutive kernel rows, on different banks)
    p->tw = strip_width(kRunPixels, g.oh, g.ow);
    p->nr = kRunPixels / p->tw + g.r - 1, p->wp = p->tw + g.s - 1;
    if (g.s == 1) p->wp |= 1;
    p->lds_bytes = tile + kRunPixels * 4 + (size_t)g.c * p->nr * p->wp * 4;
  }
  const size_t red = (size_t)p->tm * p->tn * 16 * 64 * 4;
  if (red > tile || p->lds_bytes > 64 * 1024) return false;
  p->runs_per_img = p->tw ? (int)(ceil_div(g.oh, kRunPixels / p->tw) * ceil_div(g.ow, p->tw)) : (int)ceil_div(g.P, kRunPixels);
  const int64_t total = (int64_t)g.n * p->runs_per_img;
  if (total > 0x7fffffffLL) return false;
  p->total_runs = (int)total;
  // 64-row tiles leave room for two resident blocks per compute unit (512 in all)
  // (32-row tiles: four fit, but from 1024 runs on two runs per block measure faster - half the partial results to
  // write and add: cfg3 c1 0.032 -> 0.026 ms - while fewer runs than that are better spread one per block)
  p->runs_per_block = (int)ceil_div(total, p->tm == 2 || total >= 1024 ? 512 : 1024);
  p->blocks = (int)ceil_div(total, p->runs_per_block);
  // a spare column in the last 32-column tile carries the bias gradient along; partials are then always used
  p->bias_column = g.K % 32 != 0;
  p->partial_bytes = (size_t)p->blocks * g.M * (g.K + 1) * sizeof(float);
  return true;
}

template <int TM, int TN, typename T>
static void launch_few_cols_one(const FewColsArgs& a, const FewColsPlan& p, hipStream_t st) {
  auto kernel = filter_grad_few_cols_kernel<TM, TN, T>;
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)p.blocks), dim3(kThreads), p.lds_bytes, st, a);
}

template <int TM, typename T>
static void launch_few_cols_tn(const FewColsArgs& a, const FewColsPlan& p, hipStream_t st) {
  if (p.tn == 1) launch_few_cols_one<TM, 1, T>(a, p, st);
  else if (p.tn == 2) launch_few_cols_one<TM, 2, T>(a, p, st);
  else if (p.tn == 3) launch_few_cols_one<TM, 3, T>(a, p, st);
  else launch_few_cols_one<TM, 4, T>(a, p, st);
}

vcnn_status launch_filter_grad_few_cols(const FewColsPlan& p, int dtype, const ConvGeom& g, const void* x, const void* dy,
                                        float* dw, float* dbias, float* partial, hipStream_t st) {
  const bool with_bias = p.bias_column && dbias;
  FewColsArgs a{};
  a.x = x, a.dy = dy, a.out = (p.blocks > 1 || with_bias) ? partial : dw;
  a.Kp = (int)g.K + (with_bias ? 1 : 0);
  a.n = g.n, a.c = g.c, a.h = g.h, a.w = g.w, a.m = g.k, a.r = g.r, a.s = g.s, a.ph = g.ph, a.pw = g.pw;
  a.oh = g.oh, a.ow = g.ow, a.P = (int)g.P, a.K = (int)g.K;
  a.runs_per_img = p.runs_per_img, a.total_runs = p.total_runs, a.runs_per_block = p.runs_per_block;
  a.nr = p.nr, a.wp = p.wp;
  a.tw = p.tw, a.tiles_x = p.tw ? (int)ceil_div(g.ow, p.tw) : 0;
  if (dtype == VCNN_BF16) {
    if (p.tm == 1) launch_few_cols_tn<1, bf16>(a, p, st);
    else launch_few_cols_tn<2, bf16>(a, p, st);
  } else {
    if (p.tm == 1) launch_few_cols_tn<1, float>(a, p, st);
    else launch_few_cols_tn<2, float>(a, p, st);
  }
  if (vcnn_status e = check_launch("filter_grad_few_cols")) return e;
  if (with_bias) return launch_sum_slices_split(partial, dw, dbias, g.M, (int)g.K, p.blocks, st);
  if (p.blocks == 1) return VCNN_OK;
  return launch_sum_slices(partial, nullptr, dw, VCNN_F32, g.M * g.K, p.blocks, 1, 1, 0, st);
}

}  // namespace vcnn
