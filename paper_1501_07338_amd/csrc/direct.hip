// Direct (non-matrix-core) kernels for layers whose kernel matrix is degenerate: one to four output
// maps, or one to four input channels.  With M = 1 the product of Eq. 2 is a matrix-vector product
// and the patch matrix would be written and read once per use, so these layers are bound by memory,
// not by the matrix cores; here each block stages an input band (with its halo) in LDS once and
// every loaded value feeds up to 4 x (taps) multiply-adds from registers.
//
// All three kernels are written for the generic correlation
//     out[n][o][y][x] = sum_i sum_r sum_s wgt(o,i,r,s) * in[n][i][y + r - py][x + s - px]   (zero outside)
// so that the forward pass and the input gradient (a correlation of dy with the flipped kernels,
// i.e. phi_c^{-1} applied to the transposed product, evaluated in gather form) share them.
#include "common.h"
#include "elem.h"

namespace vcnn {

static constexpr int kThreads = 256;
static constexpr int kPx = 4;                 // consecutive output pixels per thread
static constexpr size_t kMaxLds = 64 * 1024;  // static launch limit without opting in to more
static constexpr int kFewOutWeightsPerThread = 2;  // kernels of one channel kept in LDS: up to 512 padded taps

__device__ __forceinline__ int tap_index(const DirectGeom& g, int r, int s) {
  return g.flip ? (g.r - 1 - r) * g.s + (g.s - 1 - s) : r * g.s + s;
}

// One input plane's rows [y0 - py, y0 - py + rows), columns shifted by px, on their way into an LDS tile (zero
// filled outside the image).  Elements are taken in flat tile order; load() issues all of this thread's loads
// (up to U per pass) before anything waits for them, store() writes them to the tile - so a plane costs one
// memory round trip rather than one per row, and a caller can put other work between the two halves.
template <int U>
struct PlaneRegs {
  float v[U];
  bool ok[U];
  template <typename T>
  __device__ __forceinline__ void load(const DirectGeom& g, const T* __restrict__ plane, int y0, int total, int e0) {
    const int dq = kThreads / g.twp, dr = kThreads - dq * g.twp;
    int ry = e0 / g.twp;
    int rx = e0 - ry * g.twp;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int iy = y0 + ry - g.py, ix = rx - g.px;
      ok[u] = e0 + u * kThreads < total && iy >= 0 && iy < g.ih && ix >= 0 && ix < g.iw;
      v[u] = ld(plane + (ok[u] ? (int64_t)iy * g.iw + ix : 0));
      rx += dr;
      ry += dq;
      if (rx >= g.twp) rx -= g.twp, ++ry;
    }
  }
  __device__ __forceinline__ void store(float* tile, int total, int e0) const {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (e0 + u * kThreads < total) tile[e0 + u * kThreads] = ok[u] ? v[u] : 0.f;
  }
};

template <typename T>
__device__ __forceinline__ void stage_plane(const DirectGeom& g, const T* __restrict__ plane, int y0, int rows,
                                            float* tile) {
  constexpr int U = 8;
  const int total = rows * g.twp;
  for (int e0 = threadIdx.x; e0 < total; e0 += U * kThreads) {
    PlaneRegs<U> regs;
    regs.load(g, plane, y0, total, e0);
    regs.store(tile, total, e0);
  }
}

// acc[o][j] += sum_s w_o[s] * row[j + s] for one tile row, sliding a register window along s.
template <int CO, typename T>
__device__ __forceinline__ void row_taps(const DirectGeom& g, const float* row, const T* const (&wrow)[CO],
                                         float (&acc)[CO][kPx]) {
  float x0 = row[0], x1 = row[1], x2 = row[2];
  const int S = g.s;
  const int dir = g.flip ? -1 : 1;  // flipped kernels are walked backwards
  int s = 0;
#define VCNN_TAP(XA, XB, XC, XD, SS)                 \
  _Pragma("unroll") for (int o = 0; o < CO; ++o) {   \
    const float wv = ld(wrow[o] + dir * (SS));       \
    acc[o][0] = fmaf(wv, XA, acc[o][0]);             \
    acc[o][1] = fmaf(wv, XB, acc[o][1]);             \
    acc[o][2] = fmaf(wv, XC, acc[o][2]);             \
    acc[o][3] = fmaf(wv, XD, acc[o][3]);             \
  }
  for (; s + 4 <= S; s += 4) {
    const float x3 = row[s + 3], x4 = row[s + 4], x5 = row[s + 5], x6 = row[s + 6];
    VCNN_TAP(x0, x1, x2, x3, s)
    VCNN_TAP(x1, x2, x3, x4, s + 1)
    VCNN_TAP(x2, x3, x4, x5, s + 2)
    VCNN_TAP(x3, x4, x5, x6, s + 3)
    x0 = x4, x1 = x5, x2 = x6;
  }
  for (; s < S; ++s) {
    const float x3 = row[s + 3];
    VCNN_TAP(x0, x1, x2, x3, s)
    x0 = x1, x1 = x2, x2 = x3;
  }
#undef VCNN_TAP
}

// The same with the kernel rows already in LDS in walking order (flipped when staged), padded to a multiple of
// four: one 16-byte read brings four taps, instead of one scalar load - and one wait - per tap.
template <int CO>
__device__ __forceinline__ void row_taps_lds(int S, const float* row, const float* const (&wrow)[CO],
                                             float (&acc)[CO][kPx]) {
  float x0 = row[0], x1 = row[1], x2 = row[2];
  int s = 0;
#define VCNN_TAP(XA, XB, XC, XD, WV)                 \
  _Pragma("unroll") for (int o = 0; o < CO; ++o) {   \
    const float wv = WV;                             \
    acc[o][0] = fmaf(wv, XA, acc[o][0]);             \
    acc[o][1] = fmaf(wv, XB, acc[o][1]);             \
    acc[o][2] = fmaf(wv, XC, acc[o][2]);             \
    acc[o][3] = fmaf(wv, XD, acc[o][3]);             \
  }
  for (; s + 4 <= S; s += 4) {
    const float x3 = row[s + 3], x4 = row[s + 4], x5 = row[s + 5], x6 = row[s + 6];
    float4 w4[CO];
#pragma unroll
    for (int o = 0; o < CO; ++o) w4[o] = *reinterpret_cast<const float4*>(wrow[o] + s);
    VCNN_TAP(x0, x1, x2, x3, w4[o].x)
    VCNN_TAP(x1, x2, x3, x4, w4[o].y)
    VCNN_TAP(x2, x3, x4, x5, w4[o].z)
    VCNN_TAP(x3, x4, x5, x6, w4[o].w)
    x0 = x4, x1 = x5, x2 = x6;
  }
  for (; s < S; ++s) {
    const float x3 = row[s + 3];
    VCNN_TAP(x0, x1, x2, x3, wrow[o][s])
    x0 = x1, x1 = x2, x2 = x3;
  }
#undef VCNN_TAP
}

// ---- few output maps (CO <= 4), any number of input channels -----------------------------------------
// Block = (sample, band of output rows, slice of the input channels).  Partial sums over channel
// slices go to `out` as [slice][n][co][oh][ow] when isplit > 1 and are combined by sum_slices_kernel.
// T: element type of in and w; TO: element type of out (float when out holds partial sums).
template <int CO, typename T, typename TO>
__global__ __launch_bounds__(kThreads) void direct_few_out_kernel(DirectGeom g, const T* __restrict__ in,
                                                                  const T* __restrict__ w,
                                                                  const float* __restrict__ bias,
                                                                  TO* __restrict__ out, int isplit, int relu) {
  extern __shared__ float tile[];
  int b = blockIdx.x;
  const int is = b % isplit;
  b /= isplit;
  const int band = b % g.bands;
  const int n = b / g.bands;
  const int y0 = band * g.bh;
  const int bh_eff = min(g.bh, g.oh - y0);
  const int rows = bh_eff + g.r - 1;
  const int per = (g.ci + isplit - 1) / isplit;
  const int i0 = is * per, i1 = min(g.ci, i0 + per);
  const int ty = threadIdx.x / g.groups, gx = threadIdx.x - ty * g.groups;
  const bool active = ty < bh_eff;

  float acc[CO][kPx];
#pragma unroll
  for (int o = 0; o < CO; ++o)
#pragma unroll
    for (int j = 0; j < kPx; ++j) acc[o][j] = 0.f;

  // The kernels of a channel, [CO][r][sp] with rows padded to sp = a multiple of four taps and already in walking
  // order, sit in LDS behind the two tiles (two copies as well).
  const int sp = (g.s + 3) & ~3, wfloats = CO * g.r * sp;
  const bool w_in_lds = wfloats <= kFewOutWeightsPerThread * kThreads;  // else (very tall kernels) read from global
  const int tile_floats = ((g.bh + g.r - 1) * g.twp + 3) & ~3;
  float* const wl0 = tile + 2 * tile_floats;
  struct WRegs {
    float v[kFewOutWeightsPerThread];
  };
  auto load_w = [&](int i) {  // this thread's kernel elements of channel i
    WRegs wr;
#pragma unroll
    for (int u = 0; u < kFewOutWeightsPerThread; ++u) {
      const int t = threadIdx.x + u * kThreads;
      wr.v[u] = 0.f;
      if (w_in_lds && t < wfloats) {
        const int o = t / (g.r * sp), q = t - o * g.r * sp;
        const int r = q / sp, sx = q - r * sp;
        if (sx < g.s) wr.v[u] = ld(w + (int64_t)o * g.w_so + (int64_t)i * g.w_si + tap_index(g, r, sx));
      }
    }
    return wr;
  };
  auto store_w = [&](const WRegs& wr, float* wl) {
#pragma unroll
    for (int u = 0; u < kFewOutWeightsPerThread; ++u) {
      const int t = threadIdx.x + u * kThreads;
      if (w_in_lds && t < wfloats) wl[t] = wr.v[u];
    }
  };
  auto taps_of = [&](int i, const float* t, const float* wl) {
    if (!active) return;
    for (int r = 0; r < g.r; ++r) {
      if (w_in_lds) {
        const float* wrow[CO];
#pragma unroll
        for (int o = 0; o < CO; ++o) wrow[o] = wl + (o * g.r + r) * sp;
        row_taps_lds<CO>(g.s, t + (ty + r) * g.twp + gx * kPx, wrow, acc);
      } else {
        const T* wrow[CO];
#pragma unroll
        for (int o = 0; o < CO; ++o) wrow[o] = w + (int64_t)o * g.w_so + (int64_t)i * g.w_si + tap_index(g, r, 0);
        row_taps<CO, T>(g, t + (ty + r) * g.twp + gx * kPx, wrow, acc);
      }
    }
  };
  const int total = rows * g.twp;
  const T* planes = in + (int64_t)n * g.ci * g.ih * g.iw;
  constexpr int U = 12;
  if (total <= U * kThreads) {
    // Two tiles: while the block multiplies channel i out of one, the loads of channel i + 1 are in flight and
    // land in the other.  One barrier per channel: it separates the reads of a tile from its next refill and
    // publishes the tile just filled.
    PlaneRegs<U> regs;
    regs.load(g, planes + (int64_t)i0 * g.ih * g.iw, y0, total, threadIdx.x);
    WRegs wreg = load_w(i0);
    regs.store(tile, total, threadIdx.x);
    store_w(wreg, wl0);
    for (int i = i0; i < i1; ++i) {
      const int cur = (i - i0) & 1;
      __syncthreads();
      if (i + 1 < i1) {
        regs.load(g, planes + (int64_t)(i + 1) * g.ih * g.iw, y0, total, threadIdx.x);
        wreg = load_w(i + 1);
      }
      taps_of(i, tile + cur * tile_floats, wl0 + cur * wfloats);
      if (i + 1 < i1) {
        regs.store(tile + (cur ^ 1) * tile_floats, total, threadIdx.x);
        store_w(wreg, wl0 + (cur ^ 1) * wfloats);
      }
    }
  } else {
    for (int i = i0; i < i1; ++i) {
      __syncthreads();
      stage_plane(g, planes + (int64_t)i * g.ih * g.iw, y0, rows, tile);
      store_w(load_w(i), wl0);
      __syncthreads();
      taps_of(i, tile, wl0);
    }
  }
  if (!active) return;
  const int y = y0 + ty;
#pragma unroll
  for (int o = 0; o < CO; ++o) {
    TO* dst = out + ((((int64_t)is * g.n + n) * g.co + o) * g.oh + y) * g.ow;
#pragma unroll
    for (int j = 0; j < kPx; ++j) {
      const int x = gx * kPx + j;
      if (x < g.ow) {
        float v = acc[o][j];
        if (isplit == 1) {
          if (bias) v += bias[o];
          if (relu) v = fmaxf(v, 0.f);
        }
        st(dst + x, v);
      }
    }
  }
}

// out[idx] = act(bias[map(idx)] + sum_s partial[s][idx]), slices added in ascending order with four
// independent loads in flight.
template <typename TO>
__global__ __launch_bounds__(kThreads) void sum_slices_kernel(const float* __restrict__ partial,
                                                              const float* __restrict__ bias, TO* __restrict__ out,
                                                              int64_t count, int splits, int64_t plane, int maps,
                                                              int relu) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= count) return;
  float acc = 0.f;
  int s = 0;
  for (; s + 4 <= splits; s += 4) {
    const float v0 = partial[(int64_t)s * count + i], v1 = partial[(int64_t)(s + 1) * count + i];
    const float v2 = partial[(int64_t)(s + 2) * count + i], v3 = partial[(int64_t)(s + 3) * count + i];
    acc = (((acc + v0) + v1) + v2) + v3;
  }
  for (; s < splits; ++s) acc += partial[(int64_t)s * count + i];
  if (bias) acc += bias[(i / plane) % maps];
  if (relu) acc = fmaxf(acc, 0.f);
  st(out + i, acc);
}

// The same sum for many slices of a short result: a block takes 16 consecutive output elements and 16 lanes share
// an element; lane j adds slices j, j + 16, ... in ascending order, eight loads in flight, and the 16 lane sums are
// added in lane order (32 elements x 8 lanes measured slower: the results are short, the slices many).  The order is fixed by the shape alone, so results stay
// run-to-run identical.  Returns the element's sum in the threads of lane 0.
static constexpr int kSumEl = 16, kSumLanes = kThreads / kSumEl;
__device__ __forceinline__ float sum_slices_lanes(const float* __restrict__ partial, int64_t count, int64_t i, int splits,
                                                  float (*lanes)[kSumEl + 1]) {
  const int e = threadIdx.x & (kSumEl - 1), j = threadIdx.x / kSumEl;
  float acc = 0.f;
  if (i < count) {
    int s = j;
    for (; s + 7 * kSumLanes < splits; s += 8 * kSumLanes) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(s + kSumLanes * u) * count + i];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; s < splits; s += kSumLanes) acc += partial[(int64_t)s * count + i];
  }
  lanes[j][e] = acc;
  __syncthreads();
  float total = 0.f;
  if (j == 0) {
#pragma unroll
    for (int l = 0; l < kSumLanes; ++l) total += lanes[l][e];
  }
  return total;
}

template <typename TO>
__global__ __launch_bounds__(kThreads) void sum_slices_wide_kernel(const float* __restrict__ partial,
                                                                   const float* __restrict__ bias,
                                                                   TO* __restrict__ out, int64_t count, int splits,
                                                                   int64_t plane, int maps, int relu) {
  __shared__ float lanes[kSumLanes][kSumEl + 1];
  const int64_t i = (int64_t)blockIdx.x * kSumEl + (threadIdx.x & (kSumEl - 1));
  float total = sum_slices_lanes(partial, count, i, splits, lanes);
  if (threadIdx.x >= kSumEl || i >= count) return;
  if (bias) total += bias[(i / plane) % maps];
  if (relu) total = fmaxf(total, 0.f);
  st(out + i, total);
}

// Slice sum of a [rows][cols + 1] result whose last column goes to a vector of its own (a filter gradient with
// the bias gradient riding along): same lane scheme and order as sum_slices_wide_kernel.
__global__ __launch_bounds__(kThreads) void sum_slices_split_kernel(const float* __restrict__ partial,
                                                                    float* __restrict__ main, float* __restrict__ last,
                                                                    int64_t rows, int cols, int splits) {
  __shared__ float lanes[kSumLanes][kSumEl + 1];
  const int64_t count = rows * (cols + 1);
  const int64_t i = (int64_t)blockIdx.x * kSumEl + (threadIdx.x & (kSumEl - 1));
  const float total = sum_slices_lanes(partial, count, i, splits, lanes);
  if (threadIdx.x >= kSumEl || i >= count) return;
  const int64_t r = i / (cols + 1);
  const int c = (int)(i - r * (cols + 1));
  if (c < cols) main[r * cols + c] = total;
  else last[r] = total;
}

// The same split sum for large results or few slices: one thread per element, slices in ascending order, loads of
// consecutive threads coalesced.
__global__ __launch_bounds__(kThreads) void sum_slices_split_plain_kernel(const float* __restrict__ partial,
                                                                          float* __restrict__ main,
                                                                          float* __restrict__ last, int64_t rows, int cols,
                                                                          int splits) {
  const int64_t count = rows * (cols + 1);
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= count) return;
  float acc = 0.f;
  int s = 0;
  for (; s + 4 <= splits; s += 4) {  // four independent loads in flight, added in ascending order
    const float v0 = partial[(int64_t)s * count + i], v1 = partial[(int64_t)(s + 1) * count + i];
    const float v2 = partial[(int64_t)(s + 2) * count + i], v3 = partial[(int64_t)(s + 3) * count + i];
    acc = (((acc + v0) + v1) + v2) + v3;
  }
  for (; s < splits; ++s) acc += partial[(int64_t)s * count + i];
  const int64_t r = i / (cols + 1);
  const int c = (int)(i - r * (cols + 1));
  if (c < cols) main[r * cols + c] = acc;
  else last[r] = acc;
}

vcnn_status launch_sum_slices_split(const float* partial, float* main, float* last, int64_t rows, int cols, int splits,
                                    hipStream_t st) {
  const int64_t count = rows * (cols + 1);
  if (splits < 32 || count > 65536) {
    hipLaunchKernelGGL(sum_slices_split_plain_kernel, dim3((unsigned)ceil_div(count, kThreads)), dim3(kThreads), 0, st,
                       partial, main, last, rows, cols, splits);
    return check_launch("sum_slices_split");
  }
  hipLaunchKernelGGL(sum_slices_split_kernel, dim3((unsigned)ceil_div(count, kSumEl)), dim3(kThreads), 0, st, partial, main, last,
                     rows, cols, splits);
  return check_launch("sum_slices_split");
}

vcnn_status launch_sum_slices(const float* partial, const float* bias, void* out, int out_dtype, int64_t count,
                              int splits, int64_t plane, int maps, int relu, hipStream_t st) {
  if (splits >= 32 && count <= 65536) {  // few output elements, many slices: parallelise over the slices as well
    const dim3 grid((unsigned)ceil_div(count, kSumEl)), block(kThreads);
    if (out_dtype == VCNN_BF16)
      hipLaunchKernelGGL(sum_slices_wide_kernel<bf16>, grid, block, 0, st, partial, bias, (bf16*)out, count, splits, plane,
                         maps, relu);
    else
      hipLaunchKernelGGL(sum_slices_wide_kernel<float>, grid, block, 0, st, partial, bias, (float*)out, count, splits,
                         plane, maps, relu);
    return check_launch("sum_slices_wide");
  }
  const dim3 grid((unsigned)ceil_div(count, kThreads)), block(kThreads);
  if (out_dtype == VCNN_BF16)
    hipLaunchKernelGGL(sum_slices_kernel<bf16>, grid, block, 0, st, partial, bias, (bf16*)out, count, splits, plane, maps,
                       relu);
  else
    hipLaunchKernelGGL(sum_slices_kernel<float>, grid, block, 0, st, partial, bias, (float*)out, count, splits, plane,
                       maps, relu);
  return check_launch("sum_slices");
}

// ---- few input channels (CI <= 4), any number of output maps -----------------------------------------
// Block = (sample, band, group of output maps).  All CI input bands sit in LDS; output maps are
// produced four at a time so that every LDS read feeds 16 multiply-adds.
template <int CI, typename T>
__global__ __launch_bounds__(kThreads) void direct_few_in_kernel(DirectGeom g, const T* __restrict__ in,
                                                                 const T* __restrict__ w,
                                                                 const float* __restrict__ bias,
                                                                 T* __restrict__ out, int ogroup, int ogroups,
                                                                 int relu, int dact, const T* __restrict__ dact_ref) {
  extern __shared__ float tile[];
  int b = blockIdx.x;
  const int og = b % ogroups;
  b /= ogroups;
  const int band = b % g.bands;
  const int n = b / g.bands;
  const int y0 = band * g.bh;
  const int bh_eff = min(g.bh, g.oh - y0);
  const int rows = bh_eff + g.r - 1;
  const int plane_lds = (g.bh + g.r - 1) * g.twp;
  const int ty = threadIdx.x / g.groups, gx = threadIdx.x - ty * g.groups;
  const bool active = ty < bh_eff;

#pragma unroll
  for (int i = 0; i < CI; ++i) stage_plane(g, in + ((int64_t)n * CI + i) * g.ih * g.iw, y0, rows, tile + i * plane_lds);
  __syncthreads();
  if (!active) return;

  const int o_end = min(g.co, (og + 1) * ogroup);
  const int y = y0 + ty;
  for (int o0 = og * ogroup; o0 < o_end; o0 += 4) {
    float acc[4][kPx];
#pragma unroll
    for (int o = 0; o < 4; ++o)
#pragma unroll
      for (int j = 0; j < kPx; ++j) acc[o][j] = 0.f;
#pragma unroll
    for (int i = 0; i < CI; ++i)
      for (int r = 0; r < g.r; ++r) {
        const T* wrow[4];
#pragma unroll
        for (int o = 0; o < 4; ++o)  // maps past the end reuse the last valid one; their results are dropped
          wrow[o] = w + (int64_t)min(o0 + o, g.co - 1) * g.w_so + (int64_t)i * g.w_si + tap_index(g, r, 0);
        row_taps<4, T>(g, tile + i * plane_lds + (ty + r) * g.twp + gx * kPx, wrow, acc);
      }
#pragma unroll
    for (int o = 0; o < 4; ++o) {
      if (o0 + o >= o_end) break;
      T* dst = out + (((int64_t)n * g.co + o0 + o) * g.oh + y) * g.ow;
      const float bv = bias ? bias[o0 + o] : 0.f;
#pragma unroll
      for (int j = 0; j < kPx; ++j) {
        const int x = gx * kPx + j;
        if (x < g.ow) {
          float v = acc[o][j] + bv;
          if (relu) v = fmaxf(v, 0.f);
          if (dact) v = act_grad(dact, ld(dact_ref + (dst - out) + x), v);  // sigma'(.) from the tensor of out's shape
          st(dst + x, v);
        }
      }
    }
  }
}

// ---- planning ------------------------------------------------------------------------------------------
static bool plan_bands(DirectGeom* g, int planes_in_lds, int min_pitch, size_t extra_bytes = 0) {
  g->groups = (g->ow + kPx - 1) / kPx;
  if (g->groups > kThreads) return false;
  g->twp = g->groups * kPx + g->s - 1;
  if (g->twp < min_pitch) g->twp = min_pitch;
  int bh = kThreads / g->groups;
  if (bh > g->oh) bh = g->oh;
  while (bh >= 1 && (size_t)planes_in_lds * ((bh + g->r - 1) * g->twp + 4) * sizeof(float) + extra_bytes > kMaxLds - 4096) --bh;
  if (bh < 1) return false;
  g->bh = bh;
  g->bands = (g->oh + bh - 1) / bh;
  return true;
}

bool direct_fwd_geom(const ConvGeom& c, DirectGeom* g) {
  *g = DirectGeom{};
  g->n = c.n, g->ci = c.c, g->ih = c.h, g->iw = c.w, g->co = c.k, g->oh = c.oh, g->ow = c.ow;
  g->r = c.r, g->s = c.s, g->py = c.ph, g->px = c.pw;
  g->w_so = c.K, g->w_si = (int64_t)c.r * c.s, g->flip = 0;
  return true;
}

bool direct_bwd_data_geom(const ConvGeom& c, DirectGeom* g) {
  *g = DirectGeom{};
  g->n = c.n, g->ci = c.k, g->ih = c.oh, g->iw = c.ow, g->co = c.c, g->oh = c.h, g->ow = c.w;
  g->r = c.r, g->s = c.s, g->py = c.r - 1 - c.ph, g->px = c.s - 1 - c.pw;
  g->w_so = (int64_t)c.r * c.s, g->w_si = c.K, g->flip = 1;
  return true;
}

static size_t few_out_weight_bytes(const DirectGeom& g) {
  const size_t wfloats = (size_t)g.co * g.r * ((g.s + 3) & ~3);
  return wfloats <= (size_t)kFewOutWeightsPerThread * kThreads ? 2 * wfloats * sizeof(float) : 0;
}

// Channel slices for the few-output kernel: enough blocks to fill the chip, at least 8 channels each.
static int few_out_split(const DirectGeom& g) {
  const int64_t base = (int64_t)g.n * g.bands;
  int split = (int)ceil_div(768, base);
  const int max_split = g.ci / 8 > 0 ? g.ci / 8 : 1;
  if (split > max_split) split = max_split;
  if (split < 1) split = 1;
  return split;
}

bool direct_few_out_plan(DirectGeom* g, int* isplit, size_t* partial_bytes) {
  if (g->co < 1 || g->co > 4) return false;
  // two tiles (the next channel is staged while one is multiplied out) and two copies of a channel's kernels
  if (!plan_bands(g, 2, 0, few_out_weight_bytes(*g))) return false;
  *isplit = few_out_split(*g);
  *partial_bytes = *isplit > 1 ? (size_t)*isplit * g->n * g->co * g->oh * g->ow * sizeof(float) : 0;
  return true;
}

template <typename T, typename TO>
static void launch_few_out_typed(const DirectGeom& g, int isplit, const void* in, const void* w, const float* bias,
                                 void* dst, int relu, hipStream_t st) {
  const size_t lds = 2 * (size_t)(((g.bh + g.r - 1) * g.twp + 3) & ~3) * sizeof(float) + few_out_weight_bytes(g);
  const dim3 grid((unsigned)((int64_t)g.n * g.bands * isplit)), block(kThreads);
  const T* i = (const T*)in;
  const T* k = (const T*)w;
  TO* o = (TO*)dst;
  switch (g.co) {
    case 1: hipLaunchKernelGGL((direct_few_out_kernel<1, T, TO>), grid, block, lds, st, g, i, k, bias, o, isplit, relu); break;
    case 2: hipLaunchKernelGGL((direct_few_out_kernel<2, T, TO>), grid, block, lds, st, g, i, k, bias, o, isplit, relu); break;
    case 3: hipLaunchKernelGGL((direct_few_out_kernel<3, T, TO>), grid, block, lds, st, g, i, k, bias, o, isplit, relu); break;
    default: hipLaunchKernelGGL((direct_few_out_kernel<4, T, TO>), grid, block, lds, st, g, i, k, bias, o, isplit, relu); break;
  }
}

vcnn_status launch_direct_few_out(const DirectGeom& g, int dtype, int isplit, const void* in, const void* w,
                                  const float* bias, void* out, float* partial, int relu, hipStream_t st) {
  if (dtype == VCNN_BF16) {
    if (isplit > 1) launch_few_out_typed<bf16, float>(g, isplit, in, w, bias, partial, relu, st);
    else launch_few_out_typed<bf16, bf16>(g, isplit, in, w, bias, out, relu, st);
  } else {
    launch_few_out_typed<float, float>(g, isplit, in, w, bias, isplit > 1 ? (void*)partial : out, relu, st);
  }
  if (vcnn_status s = check_launch("direct_few_out")) return s;
  if (isplit == 1) return VCNN_OK;
  return launch_sum_slices(partial, bias, out, dtype, (int64_t)g.n * g.co * g.oh * g.ow, isplit, (int64_t)g.oh * g.ow,
                           g.co, relu, st);
}

bool direct_few_in_plan(DirectGeom* g, int* ogroup) {
  if (g->ci < 1 || g->ci > 4) return false;
  if (!plan_bands(g, g->ci, 0)) return false;
  // groups of output maps: multiples of 4, enough blocks to fill the chip
  const int64_t base = (int64_t)g->n * g->bands;
  int groups_wanted = (int)ceil_div(1024, base);
  int og = (int)ceil_div(g->co, groups_wanted);
  og = (int)ceil_div(og, 4) * 4;
  if (og < 4) og = 4;
  *ogroup = og;
  return true;
}

template <typename T>
static void launch_few_in_typed(const DirectGeom& g, int ogroup, const void* in, const void* w, const float* bias,
                                void* out, int relu, hipStream_t st, int dact, const void* dact_ref) {
  const size_t lds = (size_t)g.ci * (g.bh + g.r - 1) * g.twp * sizeof(float);
  const int ogroups = (int)ceil_div(g.co, ogroup);
  const dim3 grid((unsigned)((int64_t)g.n * g.bands * ogroups)), block(kThreads);
  const T* i = (const T*)in;
  const T* k = (const T*)w;
  T* o = (T*)out;
  const T* ref = (const T*)dact_ref;
  if (!ref) dact = 0;
  switch (g.ci) {
    case 1: hipLaunchKernelGGL((direct_few_in_kernel<1, T>), grid, block, lds, st, g, i, k, bias, o, ogroup, ogroups, relu, dact, ref); break;
    case 2: hipLaunchKernelGGL((direct_few_in_kernel<2, T>), grid, block, lds, st, g, i, k, bias, o, ogroup, ogroups, relu, dact, ref); break;
    case 3: hipLaunchKernelGGL((direct_few_in_kernel<3, T>), grid, block, lds, st, g, i, k, bias, o, ogroup, ogroups, relu, dact, ref); break;
    default: hipLaunchKernelGGL((direct_few_in_kernel<4, T>), grid, block, lds, st, g, i, k, bias, o, ogroup, ogroups, relu, dact, ref); break;
  }
}

vcnn_status launch_direct_few_in(const DirectGeom& g, int dtype, int ogroup, const void* in, const void* w,
                                 const float* bias, void* out, int relu, hipStream_t st, int dact, const void* dact_ref) {
  if (dtype == VCNN_BF16) launch_few_in_typed<bf16>(g, ogroup, in, w, bias, out, relu, st, dact, dact_ref);
  else launch_few_in_typed<float>(g, ogroup, in, w, bias, out, relu, st, dact, dact_ref);
  return check_launch("direct_few_in");
}

// ---- filter gradient for degenerate channel counts ------------------------------------------------------
// dw[m][c][r][s] = sum_{n,y,x} dy[n][m][y][x] * xpad[n][c][y + r - ph][x + s - pw].
// Block = (m, c, four tap chunks, slice of the batch).  A tap chunk is 8 consecutive s at one r; each
// wave owns one chunk and its lanes sweep the pixels of the staged band, four per step, keeping the 8
// partial sums in registers.  Lanes are combined with a fixed butterfly, batch slices by the caller.
static constexpr int kTapChunk = 8;

template <typename T>
__global__ __launch_bounds__(kThreads) void direct_filter_grad_kernel(DirectGeom g, const T* __restrict__ x,
                                                                      const T* __restrict__ dy,
                                                                      float* __restrict__ partial, int tap_blocks,
                                                                      int imgs_per_slice) {
  // geometry: in = x [n][ci][ih][iw]; dy = [n][co][oh][ow]; taps r x s; py/px = padding
  extern __shared__ float lds[];
  const int sch = (g.s + kTapChunk - 1) / kTapChunk;
  const int nch = g.r * sch;
  int b = blockIdx.x;
  const int tb = b % tap_blocks;
  b /= tap_blocks;
  const int mc = b % (g.co * g.ci);
  const int slice = b / (g.co * g.ci);
  const int m = mc / g.ci, c = mc - m * g.ci;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = tb * 4 + wave;
  const bool valid = q < nch;
  const int r = valid ? q / sch : 0;
  const int s0 = valid ? (q - r * sch) * kTapChunk : 0;
  const int dyp = g.groups * kPx;  // dy band pitch
  float* xt = lds;
  float* dt = lds + (g.bh + g.r - 1) * g.twp;
  DirectGeom gd = g;  // the dy plane seen as an unpadded input plane of pitch dyp
  gd.twp = dyp, gd.py = 0, gd.px = 0, gd.ih = g.oh, gd.iw = g.ow;

  float acc[kTapChunk];
#pragma unroll
  for (int t = 0; t < kTapChunk; ++t) acc[t] = 0.f;

  const int n0 = slice * imgs_per_slice, n1 = min(g.n, n0 + imgs_per_slice);
  for (int n = n0; n < n1; ++n) {
    const T* xp = x + ((int64_t)n * g.ci + c) * g.ih * g.iw;
    const T* dp = dy + ((int64_t)n * g.co + m) * g.oh * g.ow;
    for (int band = 0; band < g.bands; ++band) {
      const int y0 = band * g.bh;
      const int bh_eff = min(g.bh, g.oh - y0);
      __syncthreads();
      stage_plane(g, xp, y0, bh_eff + g.r - 1, xt);
      stage_plane(gd, dp, y0, bh_eff, dt);  // the dy band: rows y0 + [0, bh_eff), pitch dyp, zero beyond ow
      __syncthreads();
      if (valid) {
        const int npg = bh_eff * g.groups;
        for (int pg = lane; pg < npg; pg += 64) {
          const int ty = pg / g.groups, gx = pg - ty * g.groups;
          const float* dr = dt + ty * dyp + gx * kPx;
          const float d0 = dr[0], d1 = dr[1], d2 = dr[2], d3 = dr[3];
          const float* row = xt + (ty + r) * g.twp + gx * kPx + s0;
          float xs[kTapChunk + 3];
#pragma unroll
          for (int t = 0; t < kTapChunk + 3; ++t) xs[t] = row[t];
#pragma unroll
          for (int t = 0; t < kTapChunk; ++t)
            acc[t] = fmaf(d3, xs[t + 3], fmaf(d2, xs[t + 2], fmaf(d1, xs[t + 1], fmaf(d0, xs[t], acc[t]))));
        }
      }
    }
  }
  if (!valid) return;
#pragma unroll
  for (int t = 0; t < kTapChunk; ++t) {
    float v = acc[t];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    acc[t] = v;
  }
  if (lane == 0) {
    float* dst = partial + ((int64_t)slice * g.co * g.ci + mc) * g.r * g.s + (int64_t)r * g.s + s0;
#pragma unroll
    for (int t = 0; t < kTapChunk; ++t)
      if (s0 + t < g.s) dst[t] = acc[t];
  }
}

bool direct_filter_grad_plan(const ConvGeom& c, DirectGeom* g, int* slices, size_t* partial_bytes) {
  if (!(c.k <= 4 || c.c <= 4)) return false;
  direct_fwd_geom(c, g);
  const int sch = (c.s + kTapChunk - 1) / kTapChunk;
  g->groups = (g->ow + kPx - 1) / kPx;
  const int pitch = g->groups * kPx + kTapChunk * sch - 1 + 3;  // widest window any lane reads
  g->twp = pitch;
  if (g->s * 4 < kTapChunk * sch && g->r * g->s > 16) return false;  // mostly padding taps (e.g. 121x1): not worth it
  // rows per band: as many as fit in LDS next to the dy band
  int bh = g->oh;
  auto bytes = [&](int h) { return ((size_t)(h + g->r - 1) * g->twp + (size_t)h * g->groups * kPx) * sizeof(float); };
  while (bh >= 1 && bytes(bh) > kMaxLds - 4096) --bh;
  if (bh < 1) return false;
  g->bh = bh;
  g->bands = (g->oh + bh - 1) / bh;
  const int tap_blocks = (int)ceil_div((int64_t)g->r * sch, 4);
  const int64_t base = (int64_t)c.k * c.c * tap_blocks;
  int want = (int)ceil_div(2048, base);
  if (want > c.n) want = c.n;
  if (want < 1) want = 1;
  const int per = (int)ceil_div(c.n, want);
  *slices = (int)ceil_div(c.n, per);
  *partial_bytes = *slices > 1 ? (size_t)*slices * c.M * c.K * sizeof(float) : 0;
  return true;
}

vcnn_status launch_direct_filter_grad(const DirectGeom& g, int dtype, int slices, const void* x, const void* dy,
                                      float* dw, float* partial, hipStream_t st) {
  const int sch = (g.s + kTapChunk - 1) / kTapChunk;
  const int tap_blocks = (int)ceil_div((int64_t)g.r * sch, 4);
  const int per = (int)ceil_div(g.n, slices);
  const size_t lds = ((size_t)(g.bh + g.r - 1) * g.twp + (size_t)g.bh * g.groups * kPx) * sizeof(float);
  const int64_t blocks = (int64_t)g.co * g.ci * tap_blocks * slices;
  if (blocks > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "direct filter gradient: too many blocks");
  float* dst = slices > 1 ? partial : dw;
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL(direct_filter_grad_kernel<bf16>, dim3((unsigned)blocks), dim3(kThreads), lds, st, g,
                       (const bf16*)x, (const bf16*)dy, dst, tap_blocks, per);
  else
    hipLaunchKernelGGL(direct_filter_grad_kernel<float>, dim3((unsigned)blocks), dim3(kThreads), lds, st, g,
                       (const float*)x, (const float*)dy, dst, tap_blocks, per);
  if (vcnn_status s = check_launch("direct_filter_grad")) return s;
  if (slices == 1) return VCNN_OK;
  return launch_sum_slices(partial, nullptr, dw, VCNN_F32, (int64_t)g.co * g.ci * g.r * g.s, slices, 1, 1, 0, st);
}

}  // namespace vcnn
