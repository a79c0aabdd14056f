// Implicit-unroll convolution for small layers (a few hundred MFLOP: the second layer of the small
// recognition network at batch 128).  Their cost is latency, not arithmetic: in the slab kernel a block walks
// the whole contraction K = C*R*S through a chain of fetch -> barrier -> MFMA rounds, and there are too few
// blocks to fill the chip.  Here a block owns 32 output maps x 32 consecutive output pixels of one sample and
// its 4 to 8 waves split the contraction (one wave per 64 indices).  The input rows under the pixels (all
// channels, with halo, zero padded) are staged in LDS once; every wave requests its share of the kernel-matrix
// rows from global memory before it waits for that tile, so all global latencies overlap; the B operand of
// each MFMA is then read from the tile at lane_base(pixel) + tap_offset(c, r, s) - the patch-matrix entry of
// Eq. 2 formed by address arithmetic - and the waves' partial tiles are added in wave order through LDS.
// Three barriers in all.  The input gradient runs the same kernel on dy with the flipped, channel-transposed
// kernel matrix (back-propagation paragraph of "Vectorizing Convolution"), which a small pass writes first.
#include <algorithm>

#include "common.h"
#include "elem.h"
#include "mma_core.h"

namespace vcnn {

struct SmallConvArgs {
  const void* x;      // [n][c][h][w] input of the correlation (forward: x; input gradient: dy)
  const void* wgt;    // kernel matrix [m][K], K = c*r*s, row-major
  const float* bias;  // [m] or null
  void* y;            // [n][m][oh][ow]
  int n, c, h, w, m, r, s, ph, pw, oh, ow, P;
  int K, Kp;          // c*r*s, and rounded up to a multiple of 4 (tap-table length)
  int nr, wp;         // rows and row pitch of the staged tile, per channel
  unsigned magic_plane, magic_wp;  // ceil(2^32 / (nr * wp)), ceil(2^32 / wp): division by multiply-high
  int vec_a;          // 16-byte kernel-matrix loads (K % 4 == 0, aligned)
  int relu;
  int tiles_m, tiles_per_img, kper;
};

template <typename T>
__global__ __launch_bounds__(512) void conv_small_kernel(SmallConvArgs a) {
  extern __shared__ int small_lds[];
  int* const tapoff = small_lds;                                         // [Kp]
  float* const halo = reinterpret_cast<float*>(small_lds + a.Kp);        // [c][nr][wp]
  const int plane = a.nr * a.wp;
  float* const red = reinterpret_cast<float*>(small_lds);                // [waves - 1][16][64], reuses table + tile
  const int waves = blockDim.x >> 6;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int RS = a.r * a.s;

  int b = blockIdx.x;
  const int i0 = (b % a.tiles_m) * 32;
  b /= a.tiles_m;
  const int n = b / a.tiles_per_img;
  const int p0 = (b - n * a.tiles_per_img) * 32;
  const int oh_first = p0 / a.ow;

  // tap table: offset of tap k = (cc, r, s) inside the tile; padding entries point at 0 (their columns are masked)
  for (int k = tid; k < a.Kp; k += blockDim.x) {
    int off = 0;
    if (k < a.K) {
      const int cc = k / RS, q = k - cc * RS;
      const int r = q / a.s;
      off = cc * plane + r * a.wp + (q - r * a.s);
    }
    tapoff[k] = off;
  }
  // the tile: input rows oh_first - ph + [0, nr), columns -pw + [0, wp) of every channel, zero outside the image;
  // eight loads in flight per thread, the index split with multiply-high (exact: tile size * divisor < 2^32)
  const T* xin = static_cast<const T*>(a.x) + (int64_t)n * a.c * a.h * a.w;
  const int tile_elems = a.c * plane;
  constexpr int SV = 8;
  for (int e0 = tid; e0 < tile_elems; e0 += SV * blockDim.x) {
    float v[SV];
#pragma unroll
    for (int u = 0; u < SV; ++u) {
      const int e = min(e0 + u * (int)blockDim.x, tile_elems - 1);
      const int cl = (int)__umulhi((unsigned)e, a.magic_plane), rem = e - cl * plane;
      const int ry = (int)__umulhi((unsigned)rem, a.magic_wp), rx = rem - ry * a.wp;
      const int ih = oh_first - a.ph + ry, iw = rx - a.pw;
      const bool ok = ih >= 0 && ih < a.h && iw >= 0 && iw < a.w;
      const float t = ld(xin + (ok ? (cl * a.h + ih) * a.w + iw : 0));
      v[u] = ok ? t : 0.f;
    }
#pragma unroll
    for (int u = 0; u < SV; ++u) {
      const int e = e0 + u * (int)blockDim.x;
      if (e < tile_elems) halo[e] = v[u];
    }
  }

  // this wave's share of the contraction, and the kernel-matrix row of this lane: requested now, used after the barrier
  const int i = i0 + l32;
  const bool i_ok = i < a.m;
  const T* wrow = static_cast<const T*>(a.wgt) + (int64_t)(i_ok ? i : 0) * a.K;
  const int ks = wave * a.kper, ke = min(a.K, ks + a.kper);  // kper is a multiple of 8
  constexpr int U = 8;  // groups of 8 contraction indices in flight
  float av[U][4];
  auto load_a = [&](int k0) {
#pragma unroll
    for (int g = 0; g < U; ++g) {
      const int kb = k0 + 8 * g + 4 * half;
      if (a.vec_a) {
        const bool ok = i_ok && kb < ke;  // K and the split are multiples of 4: a group of four is in or out as a whole
        const float4 t = ld4(wrow + (ok ? kb : 0));
        av[g][0] = ok ? t.x : 0.f, av[g][1] = ok ? t.y : 0.f, av[g][2] = ok ? t.z : 0.f, av[g][3] = ok ? t.w : 0.f;
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool ok = i_ok && kb + u < ke;
          const float t = ld(wrow + (ok ? kb + u : 0));
          av[g][u] = ok ? t : 0.f;
        }
      }
    }
  };
  load_a(ks);
  __syncthreads();  // table and tile are complete

  const int p = min(p0 + l32, a.P - 1);  // this lane's pixel (lanes beyond the sample's last pixel repeat it, unused)
  const int oy = p / a.ow;
  const int lane_base = (oy - oh_first) * a.wp + (p - oy * a.ow);

  f32x16 acc;
#pragma unroll
  for (int q = 0; q < 16; ++q) acc[q] = 0.f;
  for (int k0 = ks; k0 < ke; k0 += 8 * U) {
    if (k0 != ks) load_a(k0);
    float bv[U][4];
#pragma unroll
    for (int g = 0; g < U; ++g) {
      const int kb = min(k0 + 8 * g + 4 * half, a.Kp - 4);  // beyond the share: any valid entry, A is zero there
      const int4 to = *reinterpret_cast<const int4*>(tapoff + kb);
      bv[g][0] = halo[lane_base + to.x], bv[g][1] = halo[lane_base + to.y];
      bv[g][2] = halo[lane_base + to.z], bv[g][3] = halo[lane_base + to.w];
    }
#pragma unroll
    for (int g = 0; g < U; ++g)
#pragma unroll
      for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g][u], bv[g][u], acc, 0, 0, 0);
  }

  __syncthreads();  // every wave is done with the table and the tile: their memory now takes the partial tiles
  if (wave > 0) {
#pragma unroll
    for (int q = 0; q < 16; ++q) red[((wave - 1) * 16 + q) * 64 + lane] = acc[q];
  }
  __syncthreads();
  if (wave > 0) return;
  for (int w = 0; w < waves - 1; ++w)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] += red[(w * 16 + q) * 64 + lane];
  if (p0 + l32 >= a.P) return;
  T* y = static_cast<T*>(a.y);
  float bq[16];  // the bias of all 16 rows requested at once (clamped rows), not one wait per row
#pragma unroll
  for (int q = 0; q < 16; ++q) bq[q] = 0.f;
  if (a.bias) {
#pragma unroll
    for (int q = 0; q < 16; ++q) bq[q] = a.bias[min(i0 + acc_row(q, lane), a.m - 1)];
  }
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int row = i0 + acc_row(q, lane);
    if (row < a.m) {
      float v = acc[q] + bq[q];
      if (a.relu) v = fmaxf(v, 0.f);
      st(y + ((int64_t)n * a.m + row) * a.P + p, v);
    }
  }
}

static constexpr size_t kSmallLds = 112 * 1024;

// one wave per 64 contraction indices, 4 to 8 of them (more waves cost more LDS for the partial tiles than
// their shorter shares save)
static int small_waves(int64_t K) { return (int)std::min<int64_t>(8, std::max<int64_t>(4, ceil_div(K, 64))); }

static size_t small_lds_bytes(int c, int w, int r, int s, int ph, int pw, int64_t K, int* nr_out, int* wp_out) {
  const int ow = w + 2 * pw - s + 1;
  const int nr = (32 + ow - 2) / ow + 1 + r - 1, wp = w + 2 * pw;  // rows a run of 32 pixels can touch, plus halo
  *nr_out = nr, *wp_out = wp;
  const int64_t Kp = (K + 3) & ~(int64_t)3;
  const int64_t tile = ((int64_t)c * nr * wp + 3) & ~(int64_t)3;
  return std::max((size_t)(Kp + tile) * 4, (size_t)(small_waves(K) - 1) * 16 * 64 * sizeof(float));
}

// Small enough that latency, not arithmetic, is the cost: at most 768 tiles and 2^29 multiply-adds; the
// contraction between 64 and 4096; tap table, tile and partial sums within the LDS of one block.
bool conv_small_applies(int n, int c, int h, int w, int m, int r, int s, int ph, int pw) {
  const int oh = h + 2 * ph - r + 1, ow = w + 2 * pw - s + 1;
  if (oh <= 0 || ow <= 0 || w + 2 * pw < 2) return false;  // (a one-column tile has no 32-bit reciprocal)
  const int64_t K = (int64_t)c * r * s, P = (int64_t)oh * ow;
  if (K < 64 || K > 4096) return false;
  if ((int64_t)c * h * w > 0x7fffffffLL || (int64_t)m * P > 0x7fffffffLL) return false;
  int nr, wp;
  if (small_lds_bytes(c, w, r, s, ph, pw, K, &nr, &wp) > kSmallLds) return false;
  if ((int64_t)c * nr * wp > 16384) return false;  // the tile is staged in one round: keep it small
  const int64_t tiles = ceil_div(m, 32) * n * ceil_div(P, 32);
  return tiles <= 768 && tiles * 32 * 32 * K <= ((int64_t)1 << 29);  // multiply-adds as executed, tile padding included
}

vcnn_status launch_conv_small(int dtype, int n, int c, int h, int w, int m, int r, int s, int ph, int pw, const void* x,
                              const void* wgt, const float* bias, void* y, int relu, hipStream_t st) {
  SmallConvArgs a{};
  a.x = x, a.wgt = wgt, a.bias = bias, a.y = y;
  a.n = n, a.c = c, a.h = h, a.w = w, a.m = m, a.r = r, a.s = s, a.ph = ph, a.pw = pw;
  a.oh = h + 2 * ph - r + 1, a.ow = w + 2 * pw - s + 1, a.P = a.oh * a.ow;
  a.K = c * r * s, a.Kp = (a.K + 3) & ~3;
  a.relu = relu;
  const size_t lds = small_lds_bytes(c, w, r, s, ph, pw, a.K, &a.nr, &a.wp);
  a.magic_plane = (unsigned)((((uint64_t)1 << 32) + (uint64_t)(a.nr * a.wp) - 1) / (uint64_t)(a.nr * a.wp));
  a.magic_wp = (unsigned)((((uint64_t)1 << 32) + (uint64_t)a.wp - 1) / (uint64_t)a.wp);
  a.vec_a = a.K % 4 == 0 && (dtype == VCNN_BF16 ? group_aligned<bf16>(wgt) : group_aligned<float>(wgt));
  const int waves = small_waves(a.K);
  a.kper = (int)ceil_div(ceil_div(a.K, waves), 8) * 8;
  a.tiles_m = (int)ceil_div(m, 32);
  a.tiles_per_img = (int)ceil_div(a.P, 32);
  const int64_t tiles = (int64_t)a.tiles_m * n * a.tiles_per_img;
  const dim3 grid((unsigned)tiles), block(64 * waves);
  static bool opted[2] = {false, false};
  if (dtype == VCNN_BF16) {
    if (!opted[1]) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(conv_small_kernel<bf16>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmallLds);
      opted[1] = true;
    }
    hipLaunchKernelGGL(conv_small_kernel<bf16>, grid, block, lds, st, a);
  } else {
    if (!opted[0]) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(conv_small_kernel<float>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmallLds);
      opted[0] = true;
    }
    hipLaunchKernelGGL(conv_small_kernel<float>, grid, block, lds, st, a);
  }
  return check_launch("conv_small");
}

// ---- input gradient of small layers: transposed product and phi_c^{-1} in one kernel ---------------------------
// The back-propagation paragraph of "Vectorizing Convolution" forms the patch-matrix gradient
// dcol[(c, r, s)][p] = sum_m W[m][c][r][s] dy[m][p] and folds it back with phi_c^{-1}.  For a small layer both steps
// fit on chip: a block owns one sample and four input channels (one per wave) and stages the sample's dy [m][P] in
// LDS.  The r*s rows of dcol that belong to a wave's channel are one 32-row MFMA tile (taps on the row axis, the
// sample's pixels on the column axis, maps as the contraction).  phi_c^{-1} is applied straight from the
// accumulator registers (lane = output pixel, register = tap): tap by tap, every lane adds its entry to the input
// pixel it belongs to in an h x w plane in LDS.  One such step touches distinct pixels (one tap, different output
// pixels); the two half-waves, which hold different taps, use a plane each, and the two are added at the end.  A
// wave's LDS instructions execute in program order, so every input pixel sums its taps in a fixed order and the
// result is bit-identical run to run.  Neither the patch-matrix gradient nor a flipped kernel matrix goes through
// HBM, and nothing is multiplied with the zero border of a 'valid' layer.  What such a layer costs is latency, so
// a thread requests everything it needs from global memory (its share of dy, the kernel-matrix entries of up to
// 64 maps) before it waits for any of it, and the loops over maps and taps are free of branches.
struct SmallBwdArgs {
  const void* dy;   // [n][m][oh][ow]
  const void* wgt;  // [m][c][r][s]
  void* dx;         // [n][c][h][w]
  int n, c, h, w, m, r, s, ph, pw, oh, ow, P;
  int RS;          // taps per channel (at most 32)
  int dy_floats;   // staged dy incl. its zero tail
  int chunks;      // channel groups of four
};

static constexpr int kSmallBwdWaves = 4;
static constexpr int kXcds = 8;  // block ids are dealt round-robin to the chip's 8 accelerator dies

// NT: 32-pixel tiles per sample.  WPS: waves per SIMD the registers are held to; 4 (a few values then live in
// scratch memory) only pays when the grid would otherwise not be resident at once.
template <int NT, int WPS>
__global__ __launch_bounds__(64 * kSmallBwdWaves, WPS) void conv_small_bwd_kernel(SmallBwdArgs a) {
  using T = float;  // the bf16 variant has its own matrix-core route for these layers
  constexpr int kThreads = 64 * kSmallBwdWaves;
  extern __shared__ int small_lds[];
  int* const taprs = small_lds;                                 // [32]: (r << 16) | s of tap t, -1 beyond the last tap
  float* const dyl = reinterpret_cast<float*>(small_lds + 32);  // [m][P] as in memory, then 32 zeros
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int hw = a.h * a.w;
  float* const planes = dyl + a.dy_floats + wave * 2 * hw;  // [2][h][w]: this wave's channel, one plane per half-wave
  // Consecutive block ids go to different XCDs (each with its own L2): give every XCD a contiguous range of
  // (sample, channel group) pairs, so that the groups of one sample fetch its dy through the same L2.
  const int blocks = gridDim.x, xcd = blockIdx.x % kXcds;
  const int b = xcd * (blocks / kXcds) + min(xcd, blocks % kXcds) + blockIdx.x / kXcds;
  const int n = b / a.chunks;
  const int c = (b - n * a.chunks) * kSmallBwdWaves + wave;
  const bool c_ok = c < a.c;  // a wave without a channel runs along on channel 0 and stores nothing

  // A operand: row = tap t of this wave's channel, contraction index = map
  const bool t_ok = l32 < a.RS;
  const T* const wgt = static_cast<const T*>(a.wgt);
  const int wstride = a.c * a.RS;  // between maps; the whole kernel tensor is below 2^31 elements
  const int woff = (c_ok ? c : 0) * a.RS + (t_ok ? l32 : 0) + half * wstride;
  constexpr int U = 32;  // MFMA steps (two maps each) per batch of loads
  float av[U];
  auto load_a = [&](int k0) {
#pragma unroll
    for (int g = 0; g < U; ++g) {
      const int k = k0 + 2 * g + half;
      const float t = ld(wgt + woff + min(k0 + 2 * g, a.m - 1 - half) * wstride);  // beyond the last map: a valid address
      av[g] = t_ok && k < a.m ? t : 0.f;
    }
  };
  load_a(0);

  // the sample's dy, a straight copy, sixteen loads in flight per thread
  const T* dyn = static_cast<const T*>(a.dy) + (int64_t)n * a.m * a.P;
  const int total = a.m * a.P;
  constexpr int V = 16;
  for (int e0 = tid; e0 < a.dy_floats; e0 += V * kThreads) {
    float v[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const int e = e0 + u * kThreads;
      v[u] = e < total ? ld(dyn + e) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const int e = e0 + u * kThreads;
      if (e < a.dy_floats) dyl[e] = v[u];
    }
  }
  if (tid < 32) {
    const int r = tid / a.s;
    taprs[tid] = tid < a.RS ? (r << 16) | (tid - r * a.s) : -1;
  }
  for (int j = lane; j < 2 * hw; j += 64) planes[j] = 0.f;
  __syncthreads();

  f32x16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;
  // In groups of four steps (one branch per group); steps beyond the last map multiply a zero A.  Columns beyond P
  // of the last tile read into the next map's row (or the zeros): finite, and never used.
  for (int k0 = 0; k0 < a.m; k0 += 2 * U) {
    if (k0) load_a(k0);
#pragma unroll
    for (int g0 = 0; g0 < U; g0 += 4) {
      if (k0 + 2 * g0 < a.m) {
        float bv[4][NT];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int k = min(k0 + 2 * (g0 + g) + half, a.m - 1);
#pragma unroll
          for (int j = 0; j < NT; ++j) bv[g][j] = dyl[k * a.P + l32 + 32 * j];
        }
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int j = 0; j < NT; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g0 + g], bv[g][j], acc[j], 0, 0, 0);
      }
    }
  }

  // phi_c^{-1}: tap (r, s) of output pixel (oy, ox) belongs to input pixel (oy - ph + r, ox - pw + s)
  float* const plane = planes + half * hw;
  int y0[NT], x0[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int p = 32 * j + l32;
    const int oy = p / a.ow;
    y0[j] = p < a.P ? oy - a.ph : -(1 << 20);  // a pixel beyond the sample's last one lands outside the plane
    x0[j] = p - oy * a.ow - a.pw;
  }
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int rs = taprs[acc_row(q, lane)];
    int idx[NT];
    bool ok[NT];
    float old[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int y = y0[j] + (rs >> 16), x = x0[j] + (rs & 0xffff);
      ok[j] = rs >= 0 && (unsigned)y < (unsigned)a.h && (unsigned)x < (unsigned)a.w;
      idx[j] = ok[j] ? y * a.w + x : 0;
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) old[j] = plane[idx[j]];
#pragma unroll
    for (int j = 0; j < NT; ++j)
      if (ok[j]) plane[idx[j]] = old[j] + acc[j][q];
  }
  if (!c_ok) return;
  T* dxp = static_cast<T*>(a.dx) + ((int64_t)n * a.c + c) * hw;
  for (int j = lane; j < hw; j += 64) st(dxp + j, planes[j] + planes[hw + j]);
}

static constexpr size_t kSmallBwdLds = 96 * 1024;

static size_t small_bwd_layout(int m, int P, int hw, int* dy_floats) {
  *dy_floats = m * P + 32;  // the last tile's columns beyond P read on into the next row, at most 31 past the end
  return (32 + (size_t)*dy_floats + (size_t)kSmallBwdWaves * 2 * hw) * sizeof(float);
}

// At most 32 taps and 128 output pixels per sample, a few hundred MFLOP as executed, more than four input channels.
bool conv_small_bwd_applies(int dtype, int n, int c, int h, int w, int m, int r, int s, int ph, int pw) {
  const int oh = h + 2 * ph - r + 1, ow = w + 2 * pw - s + 1;
  if (dtype != VCNN_F32 || oh <= 0 || ow <= 0 || r * s > 32 || (int64_t)oh * ow > 128 || (int64_t)h * w > 1024 || c <= 4 ||
      m <= 4 || m > 4096 || (int64_t)m * c * r * s > 0x7fffffffLL)
    return false;
  int dy_floats;
  if (small_bwd_layout(m, oh * ow, h * w, &dy_floats) > kSmallBwdLds) return false;
  const int64_t blocks = (int64_t)n * ceil_div(c, kSmallBwdWaves);
  return blocks <= (1 << 16) && blocks * kSmallBwdWaves * 32 * ceil_div(oh * ow, 32) * 32 * m <= ((int64_t)1 << 29);
}

template <int NT, int WPS>
static void launch_small_bwd_one(const SmallBwdArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(conv_small_bwd_kernel<NT, WPS>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmallBwdLds);
    opted = true;
  }
  hipLaunchKernelGGL((conv_small_bwd_kernel<NT, WPS>), grid, block, lds, st, a);
}

template <int NT>
static void launch_small_bwd_nt(const SmallBwdArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
  // 256 compute units x 3 blocks are resident with 3 waves per SIMD; a larger grid (up to two pixel tiles) fits
  // better with 4
  if (NT <= 2 && grid.x > 768) launch_small_bwd_one<NT, NT <= 2 ? 4 : 2>(a, grid, block, lds, st);
  else launch_small_bwd_one<NT, NT <= 2 ? 3 : 2>(a, grid, block, lds, st);
}

vcnn_status launch_conv_small_bwd(int n, int c, int h, int w, int m, int r, int s, int ph, int pw,
                                  const void* dy, const void* wgt, void* dx, hipStream_t st) {
  SmallBwdArgs a{};
  a.dy = dy, a.wgt = wgt, a.dx = dx;
  a.n = n, a.c = c, a.h = h, a.w = w, a.m = m, a.r = r, a.s = s, a.ph = ph, a.pw = pw;
  a.oh = h + 2 * ph - r + 1, a.ow = w + 2 * pw - s + 1, a.P = a.oh * a.ow;
  a.RS = r * s;
  const size_t lds = small_bwd_layout(m, a.P, h * w, &a.dy_floats);
  a.chunks = (int)ceil_div(c, kSmallBwdWaves);
  const dim3 grid((unsigned)(n * a.chunks)), block(64 * kSmallBwdWaves);
  switch ((int)ceil_div(a.P, 32)) {
    case 1: launch_small_bwd_nt<1>(a, grid, block, lds, st); break;
    case 2: launch_small_bwd_nt<2>(a, grid, block, lds, st); break;
    case 3: launch_small_bwd_nt<3>(a, grid, block, lds, st); break;
    case 4: launch_small_bwd_nt<4>(a, grid, block, lds, st); break;
    default: return fail(VCNN_ERR_UNSUPPORTED, "conv_small_bwd: more than 128 output pixels per sample");
  }
  return check_launch("conv_small_bwd");
}

}  // namespace vcnn
