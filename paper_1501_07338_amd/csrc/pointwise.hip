// Bandwidth-bound operators around the convolution: sigma (ReLU, tanh, sigmoid), pooling (phi_p of Eq. 3 with the
// max operation and its argmax record, or the average), bias gradient, cost functions and the SGD update.
// Kernels are templates on the element type of the activation tensors (float or bf16); sums,
// comparisons and costs are computed on float values.
#include <algorithm>

#include "common.h"
#include "elem.h"

namespace vcnn {

static constexpr int kThreads = 256;

static vcnn_status grid_for(size_t work_items, unsigned* blocks) {
  const size_t b = (work_items + kThreads - 1) / kThreads;
  if (b > 0x7fffffffULL) return fail(VCNN_ERR_UNSUPPORTED, "tensor too large for one launch");
  *blocks = (unsigned)(b ? b : 1);
  return VCNN_OK;
}

// ---- ReLU ---------------------------------------------------------------------------------------
// Four elements per thread (16-byte / 8-byte accesses) when the tensors are aligned; the ragged
// tail and unaligned tensors take the scalar path.  In-place use (y == x, dx == dy) is allowed, so no
// __restrict__ here.
template <typename T>
__global__ __launch_bounds__(kThreads) void relu_fwd_kernel(size_t count, const T* x, T* y, int vec) {
  const size_t i = ((size_t)blockIdx.x * kThreads + threadIdx.x) * 4;
  if (vec && i + 3 < count) {
    float4 v = ld4(x + i);
    v.x = fmaxf(v.x, 0.f), v.y = fmaxf(v.y, 0.f), v.z = fmaxf(v.z, 0.f), v.w = fmaxf(v.w, 0.f);
    st4(y + i, v);
  } else {
    for (size_t e = i; e < count && e < i + 4; ++e) st(y + e, fmaxf(ld(x + e), 0.f));
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void relu_bwd_kernel(size_t count, const T* ref, const T* dy, T* dx, int vec) {
  const size_t i = ((size_t)blockIdx.x * kThreads + threadIdx.x) * 4;
  if (vec && i + 3 < count) {
    const float4 r = ld4(ref + i);
    float4 g = ld4(dy + i);
    g.x = r.x > 0.f ? g.x : 0.f, g.y = r.y > 0.f ? g.y : 0.f, g.z = r.z > 0.f ? g.z : 0.f, g.w = r.w > 0.f ? g.w : 0.f;
    st4(dx + i, g);
  } else {
    for (size_t e = i; e < count && e < i + 4; ++e) st(dx + e, ld(ref + e) > 0.f ? ld(dy + e) : 0.f);
  }
}

template <typename T>
static vcnn_status relu_fwd_typed(size_t count, const void* x, void* y, hipStream_t st) {
  unsigned blocks;
  if (vcnn_status s = grid_for((count + 3) / 4, &blocks)) return s;
  const int vec = group_aligned<T>(x) && group_aligned<T>(y);
  hipLaunchKernelGGL(relu_fwd_kernel<T>, dim3(blocks), dim3(kThreads), 0, st, count, (const T*)x, (T*)y, vec);
  return check_launch("relu_fwd");
}

template <typename T>
static vcnn_status relu_bwd_typed(size_t count, const void* ref, const void* dy, void* dx, hipStream_t st) {
  unsigned blocks;
  if (vcnn_status s = grid_for((count + 3) / 4, &blocks)) return s;
  const int vec = group_aligned<T>(ref) && group_aligned<T>(dy) && group_aligned<T>(dx);
  hipLaunchKernelGGL(relu_bwd_kernel<T>, dim3(blocks), dim3(kThreads), 0, st, count, (const T*)ref, (const T*)dy, (T*)dx,
                     vec);
  return check_launch("relu_bwd");
}

vcnn_status launch_relu_fwd(int dtype, size_t count, const void* x, void* y, hipStream_t st) {
  return dtype == VCNN_BF16 ? relu_fwd_typed<bf16>(count, x, y, st) : relu_fwd_typed<float>(count, x, y, st);
}

vcnn_status launch_relu_bwd(int dtype, size_t count, const void* ref, const void* dy, void* dx, hipStream_t st) {
  return dtype == VCNN_BF16 ? relu_bwd_typed<bf16>(count, ref, dy, dx, st) : relu_bwd_typed<float>(count, ref, dy, dx, st);
}

// ---- tanh / sigmoid -------------------------------------------------------------------------------
// The other sigma functions Eq. 1 names.  Forward from x; backward from the forward OUTPUT y
// (tanh' = 1 - y^2, sigmoid' = y (1 - y)).  One element per thread; in place allowed.
template <int ACT>
__device__ __forceinline__ float smooth_fwd(float x) {
  // tanhf / the logistic function in fp32; both saturate cleanly for large |x|
  return ACT == VCNN_ACT_TANH ? tanhf(x) : 1.f / (1.f + __expf(-x));
}
template <int ACT>
__device__ __forceinline__ float smooth_bwd(float y, float g) {
  return ACT == VCNN_ACT_TANH ? g * (1.f - y * y) : g * y * (1.f - y);
}

// sigma by run-time id (VCNN_ACT_*), for epilogues
__device__ __forceinline__ float act_apply(int act, float x) {
  if (act == VCNN_ACT_RELU) return fmaxf(x, 0.f);
  if (act == VCNN_ACT_TANH) return smooth_fwd<VCNN_ACT_TANH>(x);
  if (act == VCNN_ACT_SIGMOID) return smooth_fwd<VCNN_ACT_SIGMOID>(x);
  return x;
}

template <int ACT, typename T>
__global__ __launch_bounds__(kThreads) void smooth_fwd_kernel(size_t count, const T* x, T* y) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < count) st(y + i, smooth_fwd<ACT>(ld(x + i)));
}

template <int ACT, typename T>
__global__ __launch_bounds__(kThreads) void smooth_bwd_kernel(size_t count, const T* y, const T* dy, T* dx) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < count) st(dx + i, smooth_bwd<ACT>(ld(y + i), ld(dy + i)));
}

template <int ACT, typename T>
static vcnn_status smooth_typed(size_t count, const void* a, const void* dy, void* out, hipStream_t st) {
  unsigned blocks;
  if (vcnn_status s = grid_for(count, &blocks)) return s;
  if (dy)
    hipLaunchKernelGGL((smooth_bwd_kernel<ACT, T>), dim3(blocks), dim3(kThreads), 0, st, count, (const T*)a, (const T*)dy,
                       (T*)out);
  else
    hipLaunchKernelGGL((smooth_fwd_kernel<ACT, T>), dim3(blocks), dim3(kThreads), 0, st, count, (const T*)a, (T*)out);
  return check_launch("act");
}

// act = VCNN_ACT_TANH | VCNN_ACT_SIGMOID; dy == nullptr: forward (a = x), else backward (a = forward output)
vcnn_status launch_smooth_act(int act, int dtype, size_t count, const void* a, const void* dy, void* out, hipStream_t st) {
  if (act == VCNN_ACT_TANH)
    return dtype == VCNN_BF16 ? smooth_typed<VCNN_ACT_TANH, bf16>(count, a, dy, out, st)
                              : smooth_typed<VCNN_ACT_TANH, float>(count, a, dy, out, st);
  return dtype == VCNN_BF16 ? smooth_typed<VCNN_ACT_SIGMOID, bf16>(count, a, dy, out, st)
                            : smooth_typed<VCNN_ACT_SIGMOID, float>(count, a, dy, out, st);
}

// ---- average pooling ------------------------------------------------------------------------------
// phi_p with the average operation.  Forward: one thread per output element, window summed in row-major
// order.  Backward: exact transpose in gather form - one thread per input element adds dy / (window size)
// of every window that covers it, in ascending window order (for windows that tile the plane this is the
// paper's nearest-neighbour upscaling).  Plane (n, c) on blockIdx.y / z.
template <typename T>
__global__ __launch_bounds__(kThreads) void avgpool_fwd_kernel(vcnn_pool_desc d, int oh_n, int ow_n,
                                                               const T* __restrict__ x, T* __restrict__ y,
                                                               const float* __restrict__ bias, int act) {
  const int o = blockIdx.x * kThreads + threadIdx.x;
  const int64_t nc = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
  if (o >= oh_n * ow_n || nc >= (int64_t)d.n * d.c) return;
  const int oh = o / ow_n, ow = o - oh * ow_n;
  const T* xp = x + nc * d.h * d.w + (int64_t)(oh * d.stride_h) * d.w + ow * d.stride_w;
  float sum = 0.f;
  for (int i = 0; i < d.win_h; ++i)
    for (int j = 0; j < d.win_w; ++j) sum += ld(xp + i * d.w + j);
  float v = sum / (float)(d.win_h * d.win_w);
  if (bias) v += bias[nc % d.c];
  st(y + nc * oh_n * ow_n + o, act_apply(act, v));
}

template <typename T>
__global__ __launch_bounds__(kThreads) void avgpool_bwd_kernel(vcnn_pool_desc d, int oh_n, int ow_n,
                                                               const T* __restrict__ dy, T* __restrict__ dx) {
  const int pos = blockIdx.x * kThreads + threadIdx.x;
  const int64_t nc = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
  if (pos >= d.h * d.w || nc >= (int64_t)d.n * d.c) return;
  const int hi = pos / d.w, wi = pos - hi * d.w;
  int oh_lo = hi - d.win_h + 1;
  oh_lo = oh_lo > 0 ? (oh_lo + d.stride_h - 1) / d.stride_h : 0;
  const int oh_hi = min(oh_n - 1, hi / d.stride_h);
  int ow_lo = wi - d.win_w + 1;
  ow_lo = ow_lo > 0 ? (ow_lo + d.stride_w - 1) / d.stride_w : 0;
  const int ow_hi = min(ow_n - 1, wi / d.stride_w);
  const T* dp = dy + nc * oh_n * ow_n;
  float acc = 0.f;
  for (int oh = oh_lo; oh <= oh_hi; ++oh)
    for (int ow = ow_lo; ow <= ow_hi; ++ow) acc += ld(dp + oh * ow_n + ow);
  st(dx + nc * d.h * d.w + pos, acc / (float)(d.win_h * d.win_w));
}

template <typename T>
static void avgpool_typed(const vcnn_pool_desc& d, int oh, int ow, const void* src, void* dst, bool backward,
                          const float* bias, int act, hipStream_t st) {
  const int64_t planes = (int64_t)d.n * d.c;
  const unsigned gy = (unsigned)std::min<int64_t>(planes, 32768);
  const int64_t per_plane = backward ? (int64_t)d.h * d.w : (int64_t)oh * ow;
  const dim3 grid((unsigned)ceil_div(per_plane, kThreads), gy, (unsigned)ceil_div(planes, gy)), block(kThreads);
  if (backward)
    hipLaunchKernelGGL(avgpool_bwd_kernel<T>, grid, block, 0, st, d, oh, ow, (const T*)src, (T*)dst);
  else
    hipLaunchKernelGGL(avgpool_fwd_kernel<T>, grid, block, 0, st, d, oh, ow, (const T*)src, (T*)dst, bias, act);
}

vcnn_status launch_avgpool(const vcnn_pool_desc& d, int oh, int ow, const void* src, void* dst, bool backward,
                           const float* bias, int act, hipStream_t st) {
  if ((int64_t)d.n * d.c > 32768LL * 65535) return fail(VCNN_ERR_UNSUPPORTED, "pool: too many planes for one launch");
  if (d.dtype == VCNN_BF16) avgpool_typed<bf16>(d, oh, ow, src, dst, backward, bias, act, st);
  else avgpool_typed<float>(d, oh, ow, src, dst, backward, bias, act, st);
  return check_launch(backward ? "avgpool_bwd" : "avgpool_fwd");
}

// ---- max pooling --------------------------------------------------------------------------------
// Forward: one thread per output element, indexed flat over the whole (n, c, oh, ow) tensor, so that a
// block writes 1 KB-aligned runs of y and of the argmax record whatever the plane size (a block per
// plane leaves the 128-byte lines at plane boundaries shared between blocks, and such partial lines are
// expensive at HBM).  WIN / STRIDE are compile-time for the common square cases (2/2, 3/2), 0 = run-time
// values from the descriptor.  Row-major scan with a strict '>' keeps the lowest flat index among
// equal maxima.
template <typename T, int WIN, int STRIDE>
__global__ __launch_bounds__(kThreads) void pool_fwd_kernel(vcnn_pool_desc d, int oh_n, int ow_n, int64_t total,
                                                            const T* __restrict__ x, T* __restrict__ y,
                                                            int32_t* __restrict__ argmax,
                                                            const float* __restrict__ bias, int act) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int win_h = WIN ? WIN : d.win_h, win_w = WIN ? WIN : d.win_w;
  const int sh = STRIDE ? STRIDE : d.stride_h, sw = STRIDE ? STRIDE : d.stride_w;
  const int out_plane = oh_n * ow_n;
  const int64_t nc = idx / out_plane;  // plane (n, c)
  const int o = (int)(idx - nc * out_plane);
  const int oh = o / ow_n, ow = o - oh * ow_n;
  const T* xp = x + nc * d.h * d.w;
  const int h0 = oh * sh, w0 = ow * sw;
  float best = ld(xp + h0 * d.w + w0);
  int bi = h0 * d.w + w0;
  for (int i = 0; i < win_h; ++i)  // compile-time bounds in the specialised instantiations: fully unrolled
    for (int j = 0; j < win_w; ++j) {
      const int pos = (h0 + i) * d.w + w0 + j;
      const float v = ld(xp + pos);
      if (v > best) {
        best = v;
        bi = pos;
      }
    }
  // the per-map bias and sigma of the pooling layer (Eq. 3), when given
  if (bias) best += bias[nc % d.c];
  st(y + idx, act_apply(act, best));
  argmax[idx] = bi;
}

// One thread per input element of the plane: sums, in ascending window order, the gradients of the
// windows that cover it and recorded it.  Gather form, so no atomics and every dx element is written.
template <typename T, int WIN, int STRIDE>
__global__ __launch_bounds__(kThreads) void pool_bwd_kernel(vcnn_pool_desc d, int oh_n, int ow_n,
                                                            const T* __restrict__ dy,
                                                            const int32_t* __restrict__ argmax, T* __restrict__ dx,
                                                            int act, const T* __restrict__ ref) {
  const int pos = blockIdx.x * kThreads + threadIdx.x;
  if (pos >= d.h * d.w) return;
  const int win_h = WIN ? WIN : d.win_h, win_w = WIN ? WIN : d.win_w;
  const int sh = STRIDE ? STRIDE : d.stride_h, sw = STRIDE ? STRIDE : d.stride_w;
  const int hi = pos / d.w, wi = pos - hi * d.w;
  const int64_t nc = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;  // plane (n, c)
  if (nc >= (int64_t)d.n * d.c) return;
  // windows oh with oh*stride <= hi <= oh*stride + win - 1
  int oh_lo = hi - win_h + 1;
  oh_lo = oh_lo > 0 ? (oh_lo + sh - 1) / sh : 0;
  const int oh_hi = min(oh_n - 1, hi / sh);
  int ow_lo = wi - win_w + 1;
  ow_lo = ow_lo > 0 ? (ow_lo + sw - 1) / sw : 0;
  const int ow_hi = min(ow_n - 1, wi / sw);
  const int64_t base = nc * oh_n * ow_n;
  float acc = 0.f;
  if (WIN && STRIDE) {
    // at most ceil(WIN/STRIDE) windows per axis cover a pixel: visit that fixed set with a predicate so
    // that all (argmax, dy) loads are independent and in flight together
    constexpr int CAND = WIN && STRIDE ? (WIN + STRIDE - 1) / STRIDE : 1;
#pragma unroll
    for (int a = 0; a < CAND; ++a)
#pragma unroll
      for (int b = 0; b < CAND; ++b) {
        const int oh = oh_lo + a, ow = ow_lo + b;
        const bool ok = oh <= oh_hi && ow <= ow_hi;
        const int64_t o = base + (ok ? oh * ow_n + ow : 0);
        const int am = argmax[o];
        const float g = ld(dy + o);
        acc += (ok && am == pos) ? g : 0.f;
      }
  } else {
    for (int oh = oh_lo; oh <= oh_hi; ++oh)
      for (int ow = ow_lo; ow <= ow_hi; ++ow) {
        const int64_t o = base + oh * ow_n + ow;
        if (argmax[o] == pos) acc += ld(dy + o);
      }
  }
  if (act) acc = act_grad(act, ld(ref + nc * d.h * d.w + pos), acc);
  st(dx + nc * d.h * d.w + pos, acc);
}

template <typename T>
static vcnn_status pool_fwd_typed(const vcnn_pool_desc& d, int oh, int ow, const void* x, void* y, int32_t* argmax,
                                  const float* bias, int act, hipStream_t st) {
  const int64_t total = (int64_t)d.n * d.c * oh * ow;
  const int64_t blocks = ceil_div(total, kThreads);
  if (blocks > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "pool_fwd: too many outputs for one launch");
  const dim3 grid((unsigned)blocks), block(kThreads);
  const bool square = d.win_h == d.win_w && d.stride_h == d.stride_w;
  if (square && d.win_h == 2 && d.stride_h == 2)
    hipLaunchKernelGGL((pool_fwd_kernel<T, 2, 2>), grid, block, 0, st, d, oh, ow, total, (const T*)x, (T*)y, argmax, bias, act);
  else if (square && d.win_h == 3 && d.stride_h == 2)
    hipLaunchKernelGGL((pool_fwd_kernel<T, 3, 2>), grid, block, 0, st, d, oh, ow, total, (const T*)x, (T*)y, argmax, bias, act);
  else
    hipLaunchKernelGGL((pool_fwd_kernel<T, 0, 0>), grid, block, 0, st, d, oh, ow, total, (const T*)x, (T*)y, argmax, bias, act);
  return VCNN_OK;
}

// The same gather for small planes, staged: a block takes `pb` consecutive planes, copies their dy and
// argmax records into LDS with coalesced loads (each record is needed by up to ceil(k/s)^2 input pixels)
// and then produces the dx elements of those planes from LDS, in the same window order as above.
template <typename T, int WIN, int STRIDE>
__global__ __launch_bounds__(kThreads) void pool_bwd_staged_kernel(vcnn_pool_desc d, int oh_n, int ow_n, int pb, int vec,
                                                                   const T* __restrict__ dy,
                                                                   const int32_t* __restrict__ argmax,
                                                                   T* __restrict__ dx, int act,
                                                                   const T* __restrict__ ref) {
  extern __shared__ float pool_lds[];
  const int64_t planes = (int64_t)d.n * d.c;
  const int64_t nc0 = (int64_t)blockIdx.x * pb;
  const int np = (int)min((int64_t)pb, planes - nc0);
  const int out_plane = oh_n * ow_n, in_plane = d.h * d.w;
  float* dy_s = pool_lds;
  int* am_s = reinterpret_cast<int*>(pool_lds + pb * out_plane);
  // Small planes make this kernel one of memory latency: everything a thread reads from global memory (records
  // here, the activation reference below) is requested several elements ahead of its use.
  const int recs = np * out_plane;
  for (int i0 = threadIdx.x; i0 < recs; i0 += 4 * kThreads) {
    float dv[4];
    int av[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = min(i0 + u * kThreads, recs - 1);
      dv[u] = ld(dy + nc0 * out_plane + i);
      av[u] = argmax[nc0 * out_plane + i];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kThreads;
      if (i < recs) dy_s[i] = dv[u], am_s[i] = av[u];
    }
  }
  __syncthreads();
  const int win_h = WIN ? WIN : d.win_h, win_w = WIN ? WIN : d.win_w;
  const int sh = STRIDE ? STRIDE : d.stride_h, sw = STRIDE ? STRIDE : d.stride_w;
  if (WIN && STRIDE && vec) {  // vec: rows are a multiple of 4 pixels and dx is aligned for 4-element stores
    // four consecutive pixels of a row per thread: the windows that can have recorded any of them are a
    // fixed small set, visited in ascending (row, column) order; a window's gradient goes to the pixel
    // whose index it recorded.  One 16-byte store per thread.
    constexpr int ROWS = WIN && STRIDE ? (WIN + STRIDE - 1) / STRIDE : 1;
    constexpr int COLS = WIN && STRIDE ? (WIN + 2) / STRIDE + 1 : 1;
    const int wq = d.w / 4, items = d.h * wq;
    // (plane, row, group of four) of item e, advanced by kThreads per pass without divisions
    const int d_pl = kThreads / items, d_rem = kThreads - d_pl * items;
    const int d_hi = d_rem / wq, d_wg = d_rem - d_hi * wq;
    int pl = threadIdx.x / items;
    int hi = (threadIdx.x - pl * items) / wq;
    int wg = threadIdx.x - pl * items - hi * wq;
    constexpr int U = 4;
    const int total4 = np * items;
    for (int e0 = threadIdx.x; e0 < total4; e0 += U * kThreads) {
      float4 yv[U];  // item e is the e-th group of four pixels of the block's planes
      if (act) {
#pragma unroll
        for (int u = 0; u < U; ++u) yv[u] = ld4(ref + nc0 * in_plane + 4 * (int64_t)min(e0 + u * kThreads, total4 - 1));
      }
#pragma unroll
      for (int u = 0; u < U; ++u, pl += d_pl, hi += d_hi, wg += d_wg) {
        if (wg >= wq) wg -= wq, ++hi;
        if (hi >= d.h) hi -= d.h, ++pl;
        if (e0 + u * kThreads >= total4) continue;
        const int w0 = wg * 4;
        int oh_lo = hi - WIN + 1;
        oh_lo = oh_lo > 0 ? (oh_lo + STRIDE - 1) / STRIDE : 0;
        const int oh_hi = min(oh_n - 1, hi / STRIDE);
        int ow_lo = w0 - WIN + 1;
        ow_lo = ow_lo > 0 ? (ow_lo + STRIDE - 1) / STRIDE : 0;
        const int ow_hi = min(ow_n - 1, (w0 + 3) / STRIDE);
        const int base = pl * out_plane, pos0 = hi * d.w + w0;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int a = 0; a < ROWS; ++a)
#pragma unroll
          for (int b = 0; b < COLS; ++b) {
            const int oh = oh_lo + a, ow = ow_lo + b;
            const bool ok = oh <= oh_hi && ow <= ow_hi;
            const int o = base + (ok ? oh * ow_n + ow : 0);
            const int j = am_s[o] - pos0;
            const float g = ok ? dy_s[o] : 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] += j == t ? g : 0.f;
          }
        const int64_t at = nc0 * in_plane + (int64_t)pl * in_plane + pos0;
        if (act) {
          const float4 y = yv[u];
          acc[0] = act_grad(act, y.x, acc[0]), acc[1] = act_grad(act, y.y, acc[1]);
          acc[2] = act_grad(act, y.z, acc[2]), acc[3] = act_grad(act, y.w, acc[3]);
        }
        st4(dx + at, make_float4(acc[0], acc[1], acc[2], acc[3]));
      }
    }
    return;
  }
  // one pixel per thread; (plane, row, column) advanced by kThreads per pass without divisions
  const int d_pl = kThreads / in_plane, d_rem = kThreads - d_pl * in_plane;
  const int d_hi = d_rem / d.w, d_wi = d_rem - d_hi * d.w;
  int pl = threadIdx.x / in_plane;
  int hi = (threadIdx.x - pl * in_plane) / d.w;
  int wi = threadIdx.x - pl * in_plane - hi * d.w;
  constexpr int U = 8;
  const int total = np * in_plane;
  for (int e0 = threadIdx.x; e0 < total; e0 += U * kThreads) {
    float rv[U];
    if (act) {
#pragma unroll
      for (int u = 0; u < U; ++u) rv[u] = ld(ref + nc0 * in_plane + min(e0 + u * kThreads, total - 1));
    }
#pragma unroll
    for (int u = 0; u < U; ++u, pl += d_pl, hi += d_hi, wi += d_wi) {
      const int e = e0 + u * kThreads;
      if (wi >= d.w) wi -= d.w, ++hi;
      if (hi >= d.h) hi -= d.h, ++pl;
      if (e >= total) continue;
      const int pos = hi * d.w + wi;
      int oh_lo = hi - win_h + 1;
      oh_lo = oh_lo > 0 ? (oh_lo + sh - 1) / sh : 0;
      const int oh_hi = min(oh_n - 1, hi / sh);
      int ow_lo = wi - win_w + 1;
      ow_lo = ow_lo > 0 ? (ow_lo + sw - 1) / sw : 0;
      const int ow_hi = min(ow_n - 1, wi / sw);
      const int base = pl * out_plane;
      float acc = 0.f;
      if (WIN && STRIDE) {
        // at most ceil(WIN/STRIDE) windows per axis cover a pixel: a fixed set, visited with a predicate
        constexpr int CAND = WIN && STRIDE ? (WIN + STRIDE - 1) / STRIDE : 1;
#pragma unroll
        for (int a = 0; a < CAND; ++a)
#pragma unroll
          for (int b = 0; b < CAND; ++b) {
            const int oh = oh_lo + a, ow = ow_lo + b;
            const bool ok = oh <= oh_hi && ow <= ow_hi;
            const int o = base + (ok ? oh * ow_n + ow : 0);
            acc += (ok && am_s[o] == pos) ? dy_s[o] : 0.f;
          }
      } else {
        for (int oh = oh_lo; oh <= oh_hi; ++oh)
          for (int ow = ow_lo; ow <= ow_hi; ++ow) {
            const int o = base + oh * ow_n + ow;
            if (am_s[o] == pos) acc += dy_s[o];
          }
      }
      if (act) acc = act_grad(act, rv[u], acc);
      st(dx + nc0 * in_plane + e, acc);
    }
  }
}

template <typename T>
static void pool_bwd_typed(const vcnn_pool_desc& d, int oh, int ow, const void* dy, const int32_t* argmax, void* dx,
                           int act, const void* ref, hipStream_t st) {
  const int64_t planes = (int64_t)d.n * d.c;
  const bool square = d.win_h == d.win_w && d.stride_h == d.stride_w;
  const int which = square && d.win_h == 2 && d.stride_h == 2 ? 2 : (square && d.win_h == 3 && d.stride_h == 2 ? 3 : 0);
  // staged form: planes per block so that a block writes about 4096 dx elements and its records fit 32 KB of LDS
  const int64_t in_plane = (int64_t)d.h * d.w, out_plane = (int64_t)oh * ow;
  int64_t pb = std::max<int64_t>(1, 4096 / in_plane);
  pb = std::min(pb, std::max<int64_t>(1, (32 * 1024) / (8 * out_plane)));
  pb = std::min(pb, planes);
  if (in_plane <= 16384 && out_plane * 8 <= 32 * 1024 && ceil_div(planes, pb) <= 0x7fffffffLL) {
    const dim3 grid((unsigned)ceil_div(planes, pb)), block(kThreads);
    const size_t lds = (size_t)pb * out_plane * 8;
    const int vec = d.w % 4 == 0 && group_aligned<T>(dx) && (!act || group_aligned<T>(ref));
    if (which == 2)
      hipLaunchKernelGGL((pool_bwd_staged_kernel<T, 2, 2>), grid, block, lds, st, d, oh, ow, (int)pb, vec, (const T*)dy, argmax, (T*)dx, act, (const T*)ref);
    else if (which == 3)
      hipLaunchKernelGGL((pool_bwd_staged_kernel<T, 3, 2>), grid, block, lds, st, d, oh, ow, (int)pb, vec, (const T*)dy, argmax, (T*)dx, act, (const T*)ref);
    else
      hipLaunchKernelGGL((pool_bwd_staged_kernel<T, 0, 0>), grid, block, lds, st, d, oh, ow, (int)pb, vec, (const T*)dy, argmax, (T*)dx, act, (const T*)ref);
    return;
  }
  const unsigned gy = (unsigned)std::min<int64_t>(planes, 32768);
  const dim3 grid((unsigned)ceil_div((int64_t)d.h * d.w, kThreads), gy, (unsigned)ceil_div(planes, gy)), block(kThreads);
  if (which == 2)
    hipLaunchKernelGGL((pool_bwd_kernel<T, 2, 2>), grid, block, 0, st, d, oh, ow, (const T*)dy, argmax, (T*)dx, act, (const T*)ref);
  else if (which == 3)
    hipLaunchKernelGGL((pool_bwd_kernel<T, 3, 2>), grid, block, 0, st, d, oh, ow, (const T*)dy, argmax, (T*)dx, act, (const T*)ref);
  else
    hipLaunchKernelGGL((pool_bwd_kernel<T, 0, 0>), grid, block, 0, st, d, oh, ow, (const T*)dy, argmax, (T*)dx, act, (const T*)ref);
}

vcnn_status launch_pool_fwd(const vcnn_pool_desc& d, int oh, int ow, const void* x, void* y, int32_t* argmax,
                            const float* bias, int act, hipStream_t st) {
  const vcnn_status rc = d.dtype == VCNN_BF16 ? pool_fwd_typed<bf16>(d, oh, ow, x, y, argmax, bias, act, st)
                                               : pool_fwd_typed<float>(d, oh, ow, x, y, argmax, bias, act, st);
  if (rc != VCNN_OK) return rc;
  return check_launch("pool_fwd");
}

vcnn_status launch_pool_bwd(const vcnn_pool_desc& d, int oh, int ow, const void* dy, const int32_t* argmax, void* dx,
                            int act, const void* ref, hipStream_t st) {
  if ((int64_t)d.n * d.c > 32768LL * 65535) return fail(VCNN_ERR_UNSUPPORTED, "pool: too many planes for one launch");
  if (d.dtype == VCNN_BF16) pool_bwd_typed<bf16>(d, oh, ow, dy, argmax, dx, act, ref, st);
  else pool_bwd_typed<float>(d, oh, ow, dy, argmax, dx, act, ref, st);
  return check_launch("pool_bwd");
}

// ---- block reduction in a fixed order --------------------------------------------------------------
template <int THREADS>
__device__ __forceinline__ float block_sum(float v, float* sm) {
  sm[threadIdx.x] = v;
  __syncthreads();
  for (int s = THREADS / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sm[threadIdx.x] += sm[threadIdx.x + s];
    __syncthreads();
  }
  const float r = sm[0];
  __syncthreads();
  return r;
}

// db[m] = sum over samples and positions of dy[n][m][p].  Stage 1: block (m, slice) sums the samples of
// its slice, four independent loads in flight per thread, then the fixed block tree; stage 2 adds the
// slices in ascending order.  With one slice stage 1 writes db directly.
template <typename T>
__global__ __launch_bounds__(kThreads) void bias_grad_kernel(int n, int M, int64_t P, int per_slice,
                                                             const T* __restrict__ dy, float* __restrict__ out) {
  __shared__ float sm[kThreads];
  const int m = blockIdx.x, slice = blockIdx.y;
  const int n0 = slice * per_slice, n1 = min(n, n0 + per_slice);
  // four samples x two positions per thread and pass: eight independent (masked) loads in flight, so a slice
  // costs a few memory round trips whatever P is
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (per_slice < 4) {  // few samples per slice: eight positions of one sample per pass instead
    for (int i = n0; i < n1; ++i) {
      const T* row = dy + ((int64_t)i * M + m) * P;
      for (int64_t p = threadIdx.x; p < P; p += 8 * kThreads) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = ld(row + (p + u * kThreads < P ? p + u * kThreads : p));
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] += p + u * kThreads < P ? v[u] : 0.f;
      }
    }
  } else
  for (int i = n0; i < n1; i += 4) {
    const T* rows[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) rows[u] = dy + ((int64_t)min(i + u, n1 - 1) * M + m) * P;
    for (int64_t p = threadIdx.x; p < P; p += 2 * kThreads) {
      const bool second = p + kThreads < P;
      float v[8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        v[u] = ld(rows[u] + p);
        v[4 + u] = ld(rows[u] + (second ? p + kThreads : p));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool in = i + u < n1;
        a[u] += in ? v[u] : 0.f;
        a[4 + u] += in && second ? v[4 + u] : 0.f;
      }
    }
  }
  const float total = block_sum<kThreads>(((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7])), sm);
  if (threadIdx.x == 0) out[(int64_t)slice * M + m] = total;
}

__global__ __launch_bounds__(kThreads) void bias_grad_finish_kernel(int M, int slices, const float* __restrict__ part,
                                                                    float* __restrict__ db) {
  const int m = blockIdx.x * kThreads + threadIdx.x;
  if (m >= M) return;
  float acc = 0.f;
  for (int s = 0; s < slices; ++s) acc += part[(int64_t)s * M + m];
  db[m] = acc;
}

int bias_grad_slices(const ConvGeom& g) {
  int64_t s = ceil_div(2048, g.M);
  if (s > g.n) s = g.n;
  return (int)(s < 1 ? 1 : s);
}

size_t bias_grad_partial_bytes(const ConvGeom& g) {
  const int s = bias_grad_slices(g);
  return s > 1 ? (size_t)s * g.M * sizeof(float) : 0;
}

vcnn_status launch_bias_grad(const ConvGeom& g, int dtype, const void* dy, float* db, float* partial, hipStream_t st) {
  const int want = bias_grad_slices(g);
  const int per = (int)ceil_div(g.n, want);
  const int slices = (int)ceil_div(g.n, per);
  float* out = slices > 1 ? partial : db;
  const dim3 grid((unsigned)g.M, (unsigned)slices), block(kThreads);
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL(bias_grad_kernel<bf16>, grid, block, 0, st, g.n, (int)g.M, g.P, per, (const bf16*)dy, out);
  else
    hipLaunchKernelGGL(bias_grad_kernel<float>, grid, block, 0, st, g.n, (int)g.M, g.P, per, (const float*)dy, out);
  if (vcnn_status s = check_launch("bias_grad")) return s;
  if (slices == 1) return VCNN_OK;
  hipLaunchKernelGGL(bias_grad_finish_kernel, dim3((unsigned)ceil_div(g.M, kThreads)), block, 0, st, (int)g.M, slices,
                     partial, db);
  return check_launch("bias_grad_finish");
}

// out[c] = sum_r a[r][c]  (fully connected bias gradient): one thread per column, rows in order.
template <typename T>
__global__ __launch_bounds__(kThreads) void col_sum_kernel(int rows, int cols, const T* __restrict__ a,
                                                           float* __restrict__ out) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= cols) return;
  float acc = 0.f;
  int r = 0;
  for (; r + 4 <= rows; r += 4) {  // four independent loads in flight, added in ascending order
    const float v0 = ld(a + (int64_t)r * cols + c), v1 = ld(a + (int64_t)(r + 1) * cols + c);
    const float v2 = ld(a + (int64_t)(r + 2) * cols + c), v3 = ld(a + (int64_t)(r + 3) * cols + c);
    acc = (((acc + v0) + v1) + v2) + v3;
  }
  for (; r < rows; ++r) acc += ld(a + (int64_t)r * cols + c);
  out[c] = acc;
}

vcnn_status launch_col_sum(int dtype, int rows, int cols, const void* a, float* out, hipStream_t st) {
  const dim3 grid((unsigned)ceil_div(cols, kThreads)), block(kThreads);
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL(col_sum_kernel<bf16>, grid, block, 0, st, rows, cols, (const bf16*)a, out);
  else
    hipLaunchKernelGGL(col_sum_kernel<float>, grid, block, 0, st, rows, cols, (const float*)a, out);
  return check_launch("col_sum");
}

// ---- costs --------------------------------------------------------------------------------------
// Single block: thread t handles rows t, t+256, ...; the per-row losses are combined with the fixed
// tree of block_sum.  SMALL (at most 16 classes): a row is read into registers with all its loads in flight at
// once - the kernel is one memory latency long instead of one per class - and the arithmetic is the same.
template <bool SMALL>
__global__ __launch_bounds__(kThreads) void softmax_loss_f32_kernel(int batch, int classes, const float* __restrict__ z,
                                                                    const int32_t* __restrict__ labels,
                                                                    float* __restrict__ loss, float* __restrict__ dz) {
  __shared__ float sm[kThreads];
  float acc = 0.f;
  const float inv_b = 1.f / (float)batch;
  const float kNaN = __builtin_nanf("");
  for (int b = threadIdx.x; b < batch; b += kThreads) {
    const float* zb = z + (int64_t)b * classes;
    if constexpr (SMALL) {
      constexpr int C = 16;
      float zr[C];
#pragma unroll
      for (int j = 0; j < C; ++j) zr[j] = zb[min(j, classes - 1)];
      const int lab = labels[b];
      const bool lab_ok = lab >= 0 && lab < classes;
      float m = zr[0];
#pragma unroll
      for (int j = 1; j < C; ++j) m = j < classes ? fmaxf(m, zr[j]) : m;
      float se = 0.f;
#pragma unroll
      for (int j = 0; j < C; ++j) se += j < classes ? expf(zr[j] - m) : 0.f;
      const float lse = m + logf(se);
      float zl = zr[0];
#pragma unroll
      for (int j = 1; j < C; ++j) zl = j == lab ? zr[j] : zl;
      acc += lab_ok ? lse - zl : kNaN;  // a label outside [0, classes) has no cost: the result says so
      if (dz) {
#pragma unroll
        for (int j = 0; j < C; ++j)
          if (j < classes)
            dz[(int64_t)b * classes + j] = lab_ok ? (expf(zr[j] - lse) - (j == lab ? 1.f : 0.f)) * inv_b : kNaN;
      }
    } else {
      float m = zb[0];
      for (int j = 1; j < classes; ++j) m = fmaxf(m, zb[j]);
      float se = 0.f;
      for (int j = 0; j < classes; ++j) se += expf(zb[j] - m);
      const float lse = m + logf(se);
      const int lab = labels[b];
      const bool lab_ok = lab >= 0 && lab < classes;  // never index the row with a label outside it
      acc += lab_ok ? lse - zb[lab_ok ? lab : 0] : kNaN;
      if (dz)
        for (int j = 0; j < classes; ++j)
          dz[(int64_t)b * classes + j] = lab_ok ? (expf(zb[j] - lse) - (j == lab ? 1.f : 0.f)) * inv_b : kNaN;
    }
  }
  const float total = block_sum<kThreads>(acc, sm);
  if (threadIdx.x == 0 && loss) *loss = total * inv_b;
}

vcnn_status launch_softmax_loss_f32(int batch, int classes, const float* z, const int32_t* labels, float* loss,
                                    float* dz, hipStream_t st) {
  if (classes <= 16)
    hipLaunchKernelGGL(softmax_loss_f32_kernel<true>, dim3(1), dim3(kThreads), 0, st, batch, classes, z, labels, loss, dz);
  else
    hipLaunchKernelGGL(softmax_loss_f32_kernel<false>, dim3(1), dim3(kThreads), 0, st, batch, classes, z, labels, loss, dz);
  return check_launch("softmax_loss_f32");
}

template <typename T>
__global__ __launch_bounds__(kThreads) void l2_grad_kernel(size_t count, float inv_b, const T* __restrict__ y,
                                                           const float* __restrict__ t, T* __restrict__ dy) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < count) st(dy + i, (ld(y + i) - t[i]) * inv_b);
}

static constexpr int kL2Threads = 1024;
template <typename T>
__global__ __launch_bounds__(kL2Threads) void l2_loss_kernel(size_t count, float scale, const T* __restrict__ y,
                                                             const float* __restrict__ t, float* __restrict__ loss) {
  __shared__ float sm[kL2Threads];
  // one block (the cost has no workspace to hold partial sums): eight independent loads in flight per thread,
  // each with its own accumulator, combined in a fixed order
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  size_t i = threadIdx.x;
  for (; i + 7 * (size_t)kL2Threads < count; i += 8 * (size_t)kL2Threads) {
    float d[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) d[u] = ld(y + i + u * (size_t)kL2Threads) - t[i + u * (size_t)kL2Threads];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] += d[u] * d[u];
  }
  for (; i < count; i += kL2Threads) {
    const float d0 = ld(y + i) - t[i];
    acc[0] += d0 * d0;
  }
  const float a0 = ((acc[0] + acc[1]) + (acc[2] + acc[3])), a1 = ((acc[4] + acc[5]) + (acc[6] + acc[7]));
  const float total = block_sum<kL2Threads>(a0 + a1, sm);
  if (threadIdx.x == 0) *loss = total * scale;
}

vcnn_status launch_l2_loss(int dtype, size_t count, int batch, const void* y, const float* t, float* loss, void* dy,
                           hipStream_t st) {
  if (dy) {
    unsigned blocks;
    if (vcnn_status s = grid_for(count, &blocks)) return s;
    if (dtype == VCNN_BF16)
      hipLaunchKernelGGL(l2_grad_kernel<bf16>, dim3(blocks), dim3(kThreads), 0, st, count, 1.f / (float)batch,
                         (const bf16*)y, t, (bf16*)dy);
    else
      hipLaunchKernelGGL(l2_grad_kernel<float>, dim3(blocks), dim3(kThreads), 0, st, count, 1.f / (float)batch,
                         (const float*)y, t, (float*)dy);
    if (vcnn_status s = check_launch("l2_grad")) return s;
  }
  if (loss) {
    if (dtype == VCNN_BF16)
      hipLaunchKernelGGL(l2_loss_kernel<bf16>, dim3(1), dim3(kL2Threads), 0, st, count, 0.5f / (float)batch,
                         (const bf16*)y, t, loss);
    else
      hipLaunchKernelGGL(l2_loss_kernel<float>, dim3(1), dim3(kL2Threads), 0, st, count, 0.5f / (float)batch,
                         (const float*)y, t, loss);
    return check_launch("l2_loss");
  }
  return VCNN_OK;
}

// ---- SGD ----------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void sgd_f32_kernel(size_t count, float lr, float* __restrict__ w,
                                                           const float* __restrict__ dw) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < count) w[i] = w[i] - lr * dw[i];
}

vcnn_status launch_sgd_f32(size_t count, float lr, float* w, const float* dw, hipStream_t st) {
  unsigned blocks;
  if (vcnn_status s = grid_for(count, &blocks)) return s;
  hipLaunchKernelGGL(sgd_f32_kernel, dim3(blocks), dim3(kThreads), 0, st, count, lr, w, dw);
  return check_launch("sgd_f32");
}

// Several parameter tensors in one launch: block b works on tensor t with first[t] <= b < first[t+1].
__global__ __launch_bounds__(kThreads) void sgd_multi_kernel(SgdBatch a) {
  int t = 0;
  while (t + 1 < a.tensors && blockIdx.x >= a.first[t + 1]) ++t;
  const size_t i = (size_t)(blockIdx.x - a.first[t]) * kThreads + threadIdx.x;
  if (i >= a.count[t]) return;
  const float v = a.w[t][i] - a.lr * a.dw[t][i];
  a.w[t][i] = v;
  if (a.w16[t]) st(reinterpret_cast<bf16*>(a.w16[t]) + i, v);
}

vcnn_status launch_sgd_multi(const SgdBatch& a, hipStream_t st) {
  hipLaunchKernelGGL(sgd_multi_kernel, dim3(a.first[a.tensors]), dim3(kThreads), 0, st, a);
  return check_launch("sgd_multi");
}

// ---- bfloat16 conversion --------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void f32_to_bf16_kernel(size_t count, const float* __restrict__ src,
                                                               bf16* __restrict__ dst) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < count) st(dst + i, src[i]);
}

__global__ __launch_bounds__(kThreads) void bf16_to_f32_kernel(size_t count, const bf16* __restrict__ src,
                                                               float* __restrict__ dst) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < count) dst[i] = ld(src + i);
}

vcnn_status launch_f32_to_bf16(size_t count, const float* src, uint16_t* dst, hipStream_t st) {
  unsigned blocks;
  if (vcnn_status s = grid_for(count, &blocks)) return s;
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(blocks), dim3(kThreads), 0, st, count, src, reinterpret_cast<bf16*>(dst));
  return check_launch("f32_to_bf16");
}

vcnn_status launch_bf16_to_f32(size_t count, const uint16_t* src, float* dst, hipStream_t st) {
  unsigned blocks;
  if (vcnn_status s = grid_for(count, &blocks)) return s;
  hipLaunchKernelGGL(bf16_to_f32_kernel, dim3(blocks), dim3(kThreads), 0, st, count, reinterpret_cast<const bf16*>(src),
                     dst);
  return check_launch("bf16_to_f32");
}

}  // namespace vcnn
