// Layers with ONE output map over many input channels (the last layers of the image-to-image networks) on the
// matrix cores.  As rows of the kernel matrix such a layer has a single one, which wastes a matrix-core tile; but
// its kernel [C][R*S], read tap-major, is a perfectly good matrix with R*S rows:
//
//   forward:  Z[q][n, pixel] = sum_c w[c][q] * x[n][c][pixel]          (q = (r, s): a 1 x 1 product, R*S rows)
//             y[n][oh][ow]   = sigma(bias + sum_q Z[q][n, (oh + r - pad_h, ow + s - pad_w)])   (gather, fixed order)
//   kernel gradient:  U[q'][n, pixel] = dypad[n][pixel + q' - (R-1-pad_h, S-1-pad_w)]   (phi_c of the one-map gradient)
//             dwflip[c][q'] = sum_{n, pixel} x[n][c][pixel] * U[q'][n, pixel],   dw[c][q] = dwflip[c][R*S - 1 - q]
//
// Both are the paper's unroll + product with the roles of the short axes exchanged: the contraction of the first runs
// over the channels, that of the second over all pixels, and each executes R*S x C x (pixels of the INPUT) multiply-adds.
// The kernel-gradient product runs in the generic matrix-core kernel of gemm.hip; the forward product of layers with at
// most 64 taps has a kernel of its own here (it is bandwidth work: the input is read once, nothing is re-used from LDS).
#include "common.h"
#include "elem.h"
#include "mma_core.h"

#include <type_traits>

namespace vcnn {

static constexpr int kThreads = 256;

// y[n][oh][ow] = sigma(bias + sum over taps q = (r, s), ascending, of z[n][q][(oh + r - ph) * w + (ow + s - pw)])
template <typename T>
__global__ __launch_bounds__(kThreads) void taps_gather_kernel(const float* __restrict__ z, const float* __restrict__ bias,
                                                               T* __restrict__ y, int n, int h, int w, int r, int s, int ph,
                                                               int pw, int oh, int ow, int relu) {
  const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t total = (int64_t)n * oh * ow;
  if (e >= total) return;
  const int x0 = (int)(e % ow);
  const int64_t t = e / ow;
  const int y0 = (int)(t % oh), img = (int)(t / oh);
  const float* zi = z + (int64_t)img * r * s * h * w;
  float acc = bias ? bias[0] : 0.f;
  for (int rr = 0; rr < r; ++rr) {
    const int ih = y0 + rr - ph;
    if (ih < 0 || ih >= h) continue;
    // eight taps of the kernel row at a time: their loads are independent (clamped addresses, invalid ones
    // contribute zero) and in flight together; the sum keeps the ascending tap order
    for (int s0 = 0; s0 < s; s0 += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int ss = s0 + u, iw = x0 + ss - pw;
        const bool ok = ss < s && iw >= 0 && iw < w;
        const float t = zi[ok ? ((int64_t)(rr * s + ss) * h + ih) * w + iw : 0];
        v[u] = ok ? t : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
  }
  if (relu) acc = fmaxf(acc, 0.f);
  st(y + e, acc);
}

// Z[n][q][pixel] = sum_c w[c][q] * x[n][c][pixel] for at most 32 * TMR taps q.  A block owns 64 pixels of one sample;
// its four waves split the channels between them (so that a launch has enough waves to keep the memory busy although a
// wave holds every tap), each wave feeding the matrix cores straight from global memory: lanes 0-31 take channel
// 2 i of step i and lanes 32-63 channel 2 i + 1, a lane's B value is its pixel of that channel (128 contiguous bytes per
// half-wave) and its A values are its taps of that channel (the kernel is 32 KB per 128 channels: cache hits).  The
// loads run three batches of four steps ahead of the products.  The four partial tiles are added in wave order through
// LDS, each wave finishing and storing a quarter of the result.
static constexpr int kTapsPixels = 64, kTapsBatch = 4, kTapsRing = 4, kTapsGroups = 1, kTapsThreads = 256 * kTapsGroups;
struct __attribute__((aligned(4))) float2_dword_aligned {
  float x, y;
};

template <int TMR, typename T>
__global__ __launch_bounds__(kTapsThreads) void taps_product_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                                float* __restrict__ z, int C, int RS, int HW,
                                                                int tiles_per_img, int total_tiles) {
  constexpr int TN = kTapsPixels / 32, U = kTapsBatch;
  __shared__ float red_all[kTapsGroups][3 * TMR * TN * 16 * 64];
  // wave = K-quarter of its pixel group (one group of 64 pixels per block measures fastest: two groups side by side
  // halve the block count, and the launch then fills the compute units unevenly)
  const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3, group = tid >> 8;
  float* const red = red_all[group];
  const int l32 = lane & 31, half = lane >> 5;
  // Workgroups go to the eight XCDs in turn; each XCD takes a contiguous eighth of the tiles, so that neighbouring
  // tiles - whose rows share cache lines, the planes being aligned to nothing - meet in one second-level cache.
  const int chunk = gridDim.x / 8;  // (the grid is the tile count rounded up to a multiple of 8)
  const int tile = (blockIdx.x % 8) * chunk + blockIdx.x / 8;
  if (tile >= total_tiles) return;
  const int n = tile / tiles_per_img;
  const int px0 = (tile - n * tiles_per_img) * (kTapsPixels * kTapsGroups) + group * kTapsPixels;
  // channels per wave: an even count, so that a step's two channels belong to one wave (C is even: both have a channel
  // or neither).  The wave index is read as a scalar: the channel range, and with it the base address of every step's
  // loads, then live in scalar registers, and a load's address is that base plus a lane offset that never changes.
  const int per = (C + 7) / 8 * 2;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int c_begin = wave_s * per, c_end = min(C, c_begin + per);
  const int c_last = max(c_end - 2, 0);  // first channel of the last step with channels (fetches beyond it re-read it)
  const T* xn = x + (int64_t)n * C * HW;

  // Taps beyond RS and pixels beyond the plane are computed on clamped addresses and never stored (a row of A only
  // reaches its own row of the result, a column of B its own column), so the loads carry no condition at all; steps
  // beyond the wave's range load its last channels again and have their A values multiplied by zero.
  // float storage: a lane fetches two neighbouring pixels with one 8-byte load (at any dword boundary) and feeds them
  // to the two column tiles, i.e. column j of tile t is pixel 2 j + t of the block; bf16 storage: column j of tile t is
  // pixel 32 t + j, one 2-byte load each.
  constexpr bool PAIRS = std::is_same<T, float>::value && TN == 2;
  int px[TN], q[TMR];
  bool px_ok[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = PAIRS ? px0 + 2 * l32 + ni : px0 + ni * 32 + l32;
    px_ok[ni] = p < HW, px[ni] = min(p, HW - 1);
  }
  // where the 8-byte load starts: inside the plane (HW >= 2).  The lane whose first pixel is the last one of an odd
  // plane loads one pixel earlier and takes the second component.
  const int px_pair = min(px0 + 2 * l32, HW - 2);
  const bool pair_shifted = px0 + 2 * l32 - px_pair == 1;
  // ... and likewise two neighbouring taps with one load for the two row tiles: row j of tile t is tap 2 j + t
  constexpr bool TAP_PAIRS = std::is_same<T, float>::value && TMR == 2;
#pragma unroll
  for (int mi = 0; mi < TMR; ++mi) q[mi] = min(TAP_PAIRS ? 2 * l32 + mi : mi * 32 + l32, RS - 1);
  const int q_pair = min(2 * l32, RS - 2);  // (RS > 32 here; the lane whose first tap is the last of an odd count: as for the pixels)
  const bool q_shifted = 2 * l32 - q_pair == 1;

  f32x16 acc[TMR][TN];
  zero_acc<TMR, TN>(acc);

  // Ring of kTapsRing batches of U steps: the loads of batch b + kTapsRing - 1 are issued before the products of batch
  // b, so a load has the time of kTapsRing - 1 batches of MFMAs (of this wave and of its neighbours on the SIMD) to
  // complete.  The ring is unrolled, so that every buffer index is a constant.
  constexpr int RING = kTapsRing;
  float a_buf[RING][U][TMR], b_buf[RING][U][TN];
  int a_lane[TMR], b_lane[TN];  // element offsets of this lane's values from the first channel of a step
#pragma unroll
  for (int mi = 0; mi < TMR; ++mi) a_lane[mi] = half * RS + (TAP_PAIRS ? q_pair : q[mi]);
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) b_lane[ni] = half * HW + (PAIRS ? px_pair : px[ni]);
  auto fetch = [&](int c0, float (&ab)[U][TMR], float (&bb)[U][TN]) {  // steps (c0 - c_begin) / 2 + [0, U) of this wave
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int cs = min(c0 + 2 * i, c_last);  // scalar
      const T* const wa = w + (int64_t)cs * RS;
      const T* const xb = xn + (int64_t)cs * HW;
      if constexpr (TAP_PAIRS) {
        const float2_dword_aligned t = *reinterpret_cast<const float2_dword_aligned*>(wa + a_lane[0]);
        ab[i][0] = t.x, ab[i][1] = t.y;  // (a shifted lane picks its component when the values are used: a select
                                         // here would wait for the load on the spot)
      } else {
#pragma unroll
        for (int mi = 0; mi < TMR; ++mi) ab[i][mi] = ld(wa + a_lane[mi]);
      }
      if constexpr (PAIRS) {
        const float2_dword_aligned t = *reinterpret_cast<const float2_dword_aligned*>(xb + b_lane[0]);
        bb[i][0] = t.x, bb[i][1] = t.y;
      } else {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) bb[i][ni] = ld(xb + b_lane[ni]);
      }
    }
  };
#pragma unroll
  for (int j = 0; j < RING - 1; ++j) fetch(c_begin + j * 2 * U, a_buf[j], b_buf[j]);
  // (whole rings only, with no branch between the batches of a ring - at a branch the compiler waits for every load in
  // flight, which takes the lead away; batches beyond the wave's channels multiply zeros)
  for (int c0 = c_begin; c0 < c_end; c0 += RING * 2 * U) {
#pragma unroll
    for (int j = 0; j < RING; ++j) {
      const int cb = c0 + j * 2 * U;  // first channel of this batch
      fetch(cb + (RING - 1) * 2 * U, a_buf[(j + RING - 1) % RING], b_buf[(j + RING - 1) % RING]);
      // (the loads stay where they are issued: left to itself the scheduler moves them down to their first use, three
      // batches later, and waits for them there)
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < U; ++i) {
        const float keep = cb + 2 * i < c_end ? 1.f : 0.f;  // (scalar)
        float av[TMR], bv[TN];
#pragma unroll
        for (int mi = 0; mi < TMR; ++mi) av[mi] = keep * a_buf[j][i][mi];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) bv[ni] = b_buf[j][i][ni];
        if constexpr (TAP_PAIRS) av[0] = q_shifted ? av[1] : av[0];
        if constexpr (PAIRS) bv[0] = pair_shifted ? bv[1] : bv[0];
#pragma unroll
        for (int mi = 0; mi < TMR; ++mi)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // The four partial tiles, added in wave order - every wave finishes and stores a quarter of the accumulator registers:
  // it leaves the other three quarters of its own partial sums in LDS for their owners, and after one barrier adds, to
  // each register it owns, the three other waves' values in ascending wave order (its own value takes its place in that
  // order), so the sum does not depend on who computes it.
  constexpr int R = TMR * TN * 16, Q = R / 4;  // accumulator registers per lane, registers a wave owns
  auto slot = [&](int owner, int j, int src) {  // src = rank of the writing wave among the three that do not own
    return ((owner * Q + j) * 3 + src) * 64 + lane;
  };
#pragma unroll
  for (int f = 0; f < R; ++f) {
    const int owner = f / Q;
    if (wave != owner) red[slot(owner, f - owner * Q, wave < owner ? wave : wave - 1)] = acc[(f / 16) / TN][(f / 16) % TN][f % 16];
  }
  __syncthreads();
  float* zn = z + (int64_t)n * RS * HW;
  auto finish = [&](auto wtag) {
    constexpr int W = decltype(wtag)::value;
#pragma unroll
    for (int j = 0; j < Q; ++j) {
      constexpr int base = W * Q;
      const int f = base + j;
      const int mi = (f / 16) / TN, ni = (f / 16) % TN, r = f % 16;
      float sum = 0.f;
#pragma unroll
      for (int src = 0; src < 4; ++src) {
        const float v = src == W ? acc[mi][ni][r] : red[slot(W, j, src < W ? src : src - 1)];
        sum = src == 0 ? v : sum + v;
      }
      const int row = TAP_PAIRS ? 2 * acc_row(r, lane) + mi : mi * 32 + acc_row(r, lane);
      if (px_ok[ni] && row < RS) zn[(int64_t)row * HW + px[ni]] = sum;
    }
  };
  if (wave == 0) finish(std::integral_constant<int, 0>{});
  else if (wave == 1) finish(std::integral_constant<int, 1>{});
  else if (wave == 2) finish(std::integral_constant<int, 2>{});
  else finish(std::integral_constant<int, 3>{});
}

template <int TMR>
static void launch_taps_product(const ConvGeom& g, int dtype, const void* x, const void* w, float* z, hipStream_t st) {
  const int HW = g.h * g.w, tiles = (int)ceil_div(HW, kTapsPixels * kTapsGroups);
  const int total = g.n * tiles;
  const dim3 grid((unsigned)(ceil_div(total, 8) * 8)), block(kTapsThreads);
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL((taps_product_kernel<TMR, bf16>), grid, block, 0, st, (const bf16*)x, (const bf16*)w, z, g.c, g.r * g.s,
                       HW, tiles, total);
  else
    hipLaunchKernelGGL((taps_product_kernel<TMR, float>), grid, block, 0, st, (const float*)x, (const float*)w, z, g.c,
                       g.r * g.s, HW, tiles, total);
}

bool conv_taps_applies(const ConvGeom& g) {
  // one map, enough channels for the contraction of the forward product, enough taps for its rows
  return g.k == 1 && g.c >= 32 && g.r * g.s >= 16 && g.r * g.s <= 1024 && g.r - 1 - g.ph >= 0 && g.s - 1 - g.pw >= 0 &&
         (int64_t)g.n * g.h * g.w <= 0x7fffffffLL;
}

size_t conv_taps_fwd_bytes(const ConvGeom& g) { return (size_t)g.n * g.r * g.s * g.h * g.w * sizeof(float); }

vcnn_status launch_conv_taps_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, const float* bias, void* y,
                                 int relu, float* z, hipStream_t st) {
  const int RS = g.r * g.s, HW = g.h * g.w;
  if (RS <= 64 && g.c >= 128 && g.c % 2 == 0 && HW >= 2 && (int64_t)g.n * ceil_div(HW, kTapsPixels) <= 0x7ffffff0LL) {
    if (RS <= 32) launch_taps_product<1>(g, dtype, x, w, z, st);
    else launch_taps_product<2>(g, dtype, x, w, z, st);
    if (vcnn_status s = check_launch("taps_product")) return s;
  } else {
    GemmArgs a{};
    a.A = w, a.B = x, a.C = z, a.bias = nullptr;
    a.in_dtype = dtype, a.out_dtype = VCNN_F32;
    a.M = RS, a.N = g.n * HW, a.K = g.c;
    a.a_si = 1, a.a_sk = RS;                                     // A(q, c) = w[c][q]
    a.b_sk = HW, a.b_sj = 1, a.b_P = HW, a.b_simg = (int64_t)g.c * HW;  // B(c, (n, pixel)) = x[n][c][pixel]
    a.c_si = HW, a.c_sj = 1, a.c_P = HW, a.c_simg = (int64_t)RS * HW;   // Z[n][q][pixel]
    if (vcnn_status s = launch_gemm_f32(a, st)) return s;
  }
  const int64_t total = (int64_t)g.n * g.oh * g.ow;
  const dim3 grid((unsigned)ceil_div(total, kThreads)), block(kThreads);
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL(taps_gather_kernel<bf16>, grid, block, 0, st, z, bias, (bf16*)y, g.n, g.h, g.w, g.r, g.s, g.ph, g.pw,
                       g.oh, g.ow, relu);
  else
    hipLaunchKernelGGL(taps_gather_kernel<float>, grid, block, 0, st, z, bias, (float*)y, g.n, g.h, g.w, g.r, g.s, g.ph, g.pw,
                       g.oh, g.ow, relu);
  return check_launch("taps_gather");
}

// geometry of phi_c applied to the one-map gradient: an oh x ow "image", R x S patches, padded so that there is one
// patch per INPUT pixel
static ConvGeom unrolled_gradient_geom(const ConvGeom& g) {
  ConvGeom u{};
  u.n = g.n, u.c = 1, u.h = g.oh, u.w = g.ow, u.k = 1, u.r = g.r, u.s = g.s;
  u.ph = g.r - 1 - g.ph, u.pw = g.s - 1 - g.pw;
  u.oh = g.h, u.ow = g.w;
  u.P = (int64_t)g.h * g.w;
  u.M = 1, u.K = (int64_t)g.r * g.s, u.N = (int64_t)g.n * u.P;
  return u;
}
// the product dwflip[c][q'] = sum_j x(c, j) U[q'][j] in the terms of the kernel-gradient product of gemm.hip
static ConvGeom taps_product_geom(const ConvGeom& g) {
  ConvGeom p{};
  p.n = g.n;
  p.P = (int64_t)g.h * g.w;
  p.M = g.c, p.K = (int64_t)g.r * g.s, p.N = (int64_t)g.n * p.P;
  return p;
}

static size_t align256b(size_t b) { return (b + 255) & ~(size_t)255; }

size_t conv_taps_filter_bytes(const ConvGeom& g, int dtype) {
  const size_t esize = dtype == VCNN_BF16 ? 2 : 4;
  return align256b((size_t)g.r * g.s * g.n * g.h * g.w * esize) + align256b(bwd_filter_partial_bytes(taps_product_geom(g))) +
         align256b((size_t)g.c * g.r * g.s * sizeof(float));
}

vcnn_status launch_conv_taps_filter(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* workspace,
                                    hipStream_t st) {
  const size_t esize = dtype == VCNN_BF16 ? 2 : 4;
  const ConvGeom ug = unrolled_gradient_geom(g), pg = taps_product_geom(g);
  char* ws = (char*)workspace;
  void* u = ws;
  float* partial = (float*)(ws + align256b((size_t)g.r * g.s * g.n * g.h * g.w * esize));
  float* flipped = (float*)((char*)partial + align256b(bwd_filter_partial_bytes(pg)));
  if (vcnn_status s = launch_im2col(ug, dtype, dy, u, st)) return s;
  // "dy" of that product is x: rows = channels, sample-major [n][c][pixel]; its "patch matrix" is U
  if (vcnn_status s = launch_bwd_filter_gemm_f32(pg, dtype, x, u, nullptr, flipped, partial, st)) return s;
  return launch_flip_transpose(VCNN_F32, flipped, dw, 1, g.c, g.r * g.s, st);  // one map: a pure reversal of the taps
}

}  // namespace vcnn
