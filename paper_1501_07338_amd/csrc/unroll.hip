// phi_c and phi_c^{-1}: the unroll of the input into the dense patch matrix and its many-to-one
// inverse (Eq. 2 / Eq. 4 and the back-propagation paragraph of "Vectorizing Convolution").
//
// Patch matrix layout: row (c*R+r)*S+s, column (n*OH+oh)*OW+ow, columns contiguous.  Both kernels
// are pure data movement bound by HBM: im2col writes K*N elements and reads the (cache-resident)
// input R*S times; col2im reads K*N elements once and writes the input-sized gradient.
#include "common.h"

namespace vcnn {

static constexpr int kThreads = 256;
static constexpr int kVec = 4;  // consecutive columns per thread

// One block covers kThreads*kVec consecutive columns of one patch-matrix row.  A row (fixed c,r,s)
// is, sample by sample, a shifted window of one input plane, so consecutive columns read
// consecutive input addresses except at image-row ends.
template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) void im2col_f32_kernel(ConvGeom g, const float* __restrict__ x,
                                                              float* __restrict__ col, int chunks) {
  const int row = blockIdx.x / chunks;
  const int chunk = blockIdx.x - row * chunks;
  const int64_t j0 = ((int64_t)chunk * kThreads + threadIdx.x) * kVec;
  if (j0 >= g.N) return;
  const int c = row / (g.r * g.s);
  const int rs = row - c * (g.r * g.s);
  const int r = rs / g.s;
  const int s = rs - r * g.s;

  int n = (int)(j0 / g.P);
  int p = (int)(j0 - (int64_t)n * g.P);
  int oh = p / g.ow;
  int ow = p - oh * g.ow;

  float v[kVec];
#pragma unroll
  for (int e = 0; e < kVec; ++e) {
    const int ih = oh + r - g.ph;
    const int iw = ow + s - g.pw;
    float val = 0.f;
    if (j0 + e < g.N && ih >= 0 && ih < g.h && iw >= 0 && iw < g.w)
      val = x[(((int64_t)n * g.c + c) * g.h + ih) * g.w + iw];
    v[e] = val;
    if (++ow == g.ow) {
      ow = 0;
      if (++oh == g.oh) {
        oh = 0;
        ++n;
      }
    }
  }
  float* dst = col + (int64_t)row * g.N + j0;
  if (ALIGNED) {
    *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
#pragma unroll
    for (int e = 0; e < kVec; ++e)
      if (j0 + e < g.N) dst[e] = v[e];
  }
}

vcnn_status launch_im2col_f32(const ConvGeom& g, const float* x, float* col, hipStream_t st) {
  const int64_t chunks = ceil_div(g.N, (int64_t)kThreads * kVec);
  const int64_t blocks = chunks * g.K;
  if (blocks > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "im2col: patch matrix too large for one launch");
  const bool aligned = (g.N % kVec == 0) && ((reinterpret_cast<uintptr_t>(col) & 15) == 0);
  if (aligned)
    hipLaunchKernelGGL(im2col_f32_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, st, g, x, col, (int)chunks);
  else
    hipLaunchKernelGGL(im2col_f32_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, st, g, x, col, (int)chunks);
  return check_launch("im2col_f32");
}

// Gather form of the overlap-add: one thread per input pixel sums, in ascending (r, s) order, the
// patch-matrix entries that were copied from it.  Consecutive threads (consecutive w) read
// consecutive columns of the same row, so every patch-matrix element is read once, coalesced, and
// no atomics are needed.
__global__ __launch_bounds__(kThreads) void col2im_f32_kernel(ConvGeom g, const float* __restrict__ col,
                                                              float* __restrict__ dx, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int wi = (int)(idx % g.w);
  int64_t t = idx / g.w;
  const int hi = (int)(t % g.h);
  t /= g.h;
  const int c = (int)(t % g.c);
  const int n = (int)(t / g.c);

  float acc = 0.f;
  const int r_lo = max(0, hi + g.ph - (g.oh - 1));
  const int r_hi = min(g.r - 1, hi + g.ph);
  const int s_lo = max(0, wi + g.pw - (g.ow - 1));
  const int s_hi = min(g.s - 1, wi + g.pw);
  for (int r = r_lo; r <= r_hi; ++r) {
    const int oh = hi + g.ph - r;
    const float* rowp = col + ((int64_t)(c * g.r + r) * g.s) * g.N + (int64_t)n * g.P + (int64_t)oh * g.ow;
    for (int s = s_lo; s <= s_hi; ++s) {
      const int ow = wi + g.pw - s;
      acc += rowp[(int64_t)s * g.N + ow];
    }
  }
  dx[idx] = acc;
}

vcnn_status launch_col2im_f32(const ConvGeom& g, const float* col, float* dx, hipStream_t st) {
  const int64_t total = (int64_t)g.n * g.c * g.h * g.w;
  const int64_t blocks = ceil_div(total, kThreads);
  if (blocks > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "col2im: input too large for one launch");
  hipLaunchKernelGGL(col2im_f32_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, g, col, dx, total);
  return check_launch("col2im_f32");
}

}  // namespace vcnn
