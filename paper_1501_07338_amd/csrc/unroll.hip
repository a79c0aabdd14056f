// phi_c and phi_c^{-1}: the unroll of the input into the dense patch matrix and its many-to-one
// inverse (Eq. 2 / Eq. 4 and the back-propagation paragraph of "Vectorizing Convolution").
//
// Patch matrix layout: row (c*R+r)*S+s, column (n*OH+oh)*OW+ow, columns contiguous.  Both kernels
// are pure data movement bound by HBM: im2col writes K*N elements (the input is read once per block
// into LDS); col2im reads K*N elements once and writes the input-sized gradient.
#include "common.h"
#include "elem.h"

namespace vcnn {

static constexpr int kThreads = 256;
static constexpr int kVec = 4;  // consecutive columns per thread

// ---- phi_c --------------------------------------------------------------------------------------------
// A block owns one input plane (n, c) and a band of output rows whose pixels form a run of up to
// kThreads*kVec consecutive patch-matrix columns.  It stages the input rows of the band (plus halo,
// zero padded) in LDS with coalesced loads and then, tap by tap, writes the R*S patch-matrix rows of
// channel c for its column run: every store instruction of a wave covers 1 KB of one row.
// ALIGNED: the patch-matrix row pitch and base allow 16-byte stores.
template <bool ALIGNED, typename T>
__global__ __launch_bounds__(kThreads) void im2col_f32_kernel(ConvGeom g, const T* __restrict__ x,
                                                              T* __restrict__ col, int bh, int bands, int wp,
                                                              int rsplit) {
  extern __shared__ float tile[];
  int b = blockIdx.x;
  // kernel rows [r_begin, r_end) of this block: tall kernels are split over blocks for parallelism
  const int rpart = b % rsplit;
  b /= rsplit;
  const int rper = (g.r + rsplit - 1) / rsplit;
  const int r_begin = rpart * rper, r_end = min(g.r, r_begin + rper);
  const int band = b % bands;
  b /= bands;
  const int c = b % g.c;
  const int n = b / g.c;
  const int oh0 = band * bh;
  const int bh_eff = min(bh, g.oh - oh0);
  const int rows = bh_eff + (r_end - r_begin) - 1;  // tile row 0 = input row oh0 - ph + r_begin
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  const T* plane = x + ((int64_t)n * g.c + c) * g.h * g.w;
  for (int ry = wave; ry < rows; ry += kThreads / 64) {
    const int ih = oh0 - g.ph + r_begin + ry;
    const bool row_ok = ih >= 0 && ih < g.h;
    const T* src = plane + (int64_t)(row_ok ? ih : 0) * g.w;
    for (int rx = lane; rx < wp; rx += 64) {
      const int iw = rx - g.pw;
      const bool ok = row_ok && iw >= 0 && iw < g.w;
      const float v = ld(src + (ok ? iw : 0));
      tile[ry * wp + rx] = ok ? v : 0.f;
    }
  }
  __syncthreads();

  // This thread's runs of four consecutive columns.  Runs are aligned to multiples of four in the
  // absolute column index (shift sh), so that all but a band's first and last run are 16-byte stores.
  const int npix = bh_eff * g.ow;
  const int64_t jband = (int64_t)n * g.P + (int64_t)oh0 * g.ow;
  const int sh = ALIGNED ? (int)(jband & 3) : 0;
  for (int q0 = threadIdx.x * kVec - sh; q0 < npix; q0 += kThreads * kVec) {
    int base[kVec];
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
      const int q = min(max(q0 + e, 0), npix - 1);
      const int oy = q / g.ow;
      base[e] = oy * wp + (q - oy * g.ow);
    }
    T* dst = col + ((int64_t)(c * g.r + r_begin) * g.s) * g.N + jband + q0;
    if (ALIGNED && q0 >= 0 && q0 + kVec <= npix) {
      for (int r = 0; r < r_end - r_begin; ++r) {
        const float* t0 = tile + r * wp;
#pragma unroll 4
        for (int s = 0; s < g.s; ++s) {
          st4(dst, make_float4(t0[base[0] + s], t0[base[1] + s], t0[base[2] + s], t0[base[3] + s]));
          dst += g.N;
        }
      }
    } else {
      for (int r = 0; r < r_end - r_begin; ++r)
        for (int s = 0; s < g.s; ++s) {
          const int off = r * wp + s;
          if (q0 >= 0) st(dst, tile[base[0] + off]);
          if (q0 + 1 >= 0 && q0 + 1 < npix) st(dst + 1, tile[base[1] + off]);
          if (q0 + 2 >= 0 && q0 + 2 < npix) st(dst + 2, tile[base[2] + off]);
          if (q0 + 3 < npix) st(dst + 3, tile[base[3] + off]);
          dst += g.N;
        }
    }
  }
}

vcnn_status launch_im2col(const ConvGeom& g, int dtype, const void* x, void* col, hipStream_t st) {
  const int wp = g.w + 2 * g.pw;
  // Rows per band: at most kThreads*kVec pixels.  Kernel rows per block: all of them if the staged
  // tile (band + halo) fits 60 KB of LDS, else as many as fit; tall kernels are also split to get
  // enough blocks in flight.
  const size_t row_bytes = (size_t)wp * sizeof(float);
  const int max_rows = (int)(60 * 1024 / row_bytes);  // tile rows that fit
  if (max_rows < 1) return fail(VCNN_ERR_UNSUPPORTED, "im2col: one padded input row (%d floats) exceeds the LDS band", wp);
  int bh = (kThreads * kVec) / g.ow;
  if (bh < 1) bh = 1;  // rows wider than one pass of the block are covered by the thread loop
  if (bh > g.oh) bh = g.oh;
  if (bh > max_rows) bh = max_rows;
  const int rper_max = max_rows - bh + 1;  // >= 1
  const int bands = (int)ceil_div(g.oh, bh);
  int64_t rsplit = ceil_div(8192, (int64_t)g.n * g.c * bands);
  if (rsplit < ceil_div(g.r, rper_max)) rsplit = ceil_div(g.r, rper_max);
  if (rsplit > g.r) rsplit = g.r;
  if (rsplit < 1) rsplit = 1;
  const int rper = (int)ceil_div(g.r, rsplit);
  rsplit = ceil_div(g.r, rper);  // no empty parts
  const int64_t blocks = (int64_t)g.n * g.c * bands * rsplit;
  if (blocks > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "im2col: too many blocks for one launch");
  const size_t lds = (size_t)(bh + rper - 1) * row_bytes;
  // 16-byte stores need the row pitch to be a multiple of four elements and an aligned matrix
  const dim3 grid((unsigned)blocks), block(kThreads);
  if (dtype == VCNN_BF16) {
    const bool aligned = g.N % kVec == 0 && group_aligned<bf16>(col);
    if (aligned)
      hipLaunchKernelGGL((im2col_f32_kernel<true, bf16>), grid, block, lds, st, g, (const bf16*)x, (bf16*)col, bh, bands,
                         wp, (int)rsplit);
    else
      hipLaunchKernelGGL((im2col_f32_kernel<false, bf16>), grid, block, lds, st, g, (const bf16*)x, (bf16*)col, bh, bands,
                         wp, (int)rsplit);
  } else {
    const bool aligned = g.N % kVec == 0 && group_aligned<float>(col);
    if (aligned)
      hipLaunchKernelGGL((im2col_f32_kernel<true, float>), grid, block, lds, st, g, (const float*)x, (float*)col, bh,
                         bands, wp, (int)rsplit);
    else
      hipLaunchKernelGGL((im2col_f32_kernel<false, float>), grid, block, lds, st, g, (const float*)x, (float*)col, bh,
                         bands, wp, (int)rsplit);
  }
  return check_launch("im2col");
}

// ---- phi_c^{-1} -----------------------------------------------------------------------------------------
// Gather form of the overlap-add: one thread per input pixel sums, in ascending (r, s) order, the
// patch-matrix entries that were copied from it.  Consecutive threads (consecutive w) read
// consecutive columns of the same row, so every patch-matrix element is read once, coalesced, and
// no atomics are needed.  The tap loops run over the full kernel with a predicate instead of
// per-thread bounds, so that several independent loads are in flight per thread.
template <typename T>
__global__ __launch_bounds__(kThreads) void col2im_f32_kernel(ConvGeom g, const float* __restrict__ col,
                                                              T* __restrict__ dx, int64_t total) {
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
  for (int r = r_lo; r <= r_hi; ++r) {
    const int oh = hi + g.ph - r;
    const float* rowp = col + ((int64_t)(c * g.r + r) * g.s) * g.N + (int64_t)n * g.P + (int64_t)oh * g.ow;
    int s = 0;
    for (; s + 4 <= g.s; s += 4) {
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int ow = wi + g.pw - (s + u);
        const bool ok = ow >= 0 && ow < g.ow;
        const float t2 = rowp[(int64_t)(s + u) * g.N + (ok ? ow : 0)];
        v[u] = ok ? t2 : 0.f;
      }
      acc = (((acc + v[0]) + v[1]) + v[2]) + v[3];
    }
    for (; s < g.s; ++s) {
      const int ow = wi + g.pw - s;
      if (ow >= 0 && ow < g.ow) acc += rowp[(int64_t)s * g.N + ow];
    }
  }
  st(dx + idx, acc);
}

vcnn_status launch_col2im(const ConvGeom& g, int dtype, const float* col, void* dx, hipStream_t st) {
  const int64_t total = (int64_t)g.n * g.c * g.h * g.w;
  const int64_t blocks = ceil_div(total, kThreads);
  if (blocks > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "col2im: input too large for one launch");
  if (dtype == VCNN_BF16)
    hipLaunchKernelGGL(col2im_f32_kernel<bf16>, dim3((unsigned)blocks), dim3(kThreads), 0, st, g, col, (bf16*)dx, total);
  else
    hipLaunchKernelGGL(col2im_f32_kernel<float>, dim3((unsigned)blocks), dim3(kThreads), 0, st, g, col, (float*)dx, total);
  return check_launch("col2im");
}

}  // namespace vcnn
