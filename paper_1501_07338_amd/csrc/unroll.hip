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
// A block owns one channel c and a chunk of up to kThreads*kVec consecutive patch-matrix columns.  Chunks
// are cut at multiples of 32 columns of the whole matrix row - not at image or output-row boundaries - so
// every 128-byte line of the patch matrix is written by exactly one block: lines shared between blocks
// arrive at HBM as partial writes, which cost far more than their size.  A chunk therefore may start in
// the middle of an output row and run across several images.  For every image it touches ("part") the
// block stages the input rows under its pixels (plus halo, zero padded) in LDS with coalesced loads and
// then, tap by tap, writes the R*S patch-matrix rows of channel c for its columns: every store
// instruction of a wave covers 1 KB of one row.
// ALIGNED: the patch-matrix row pitch and base allow 16-byte stores.
template <bool ALIGNED, typename T>
__global__ __launch_bounds__(kThreads) void im2col_f32_kernel(ConvGeom g, const T* __restrict__ x,
                                                              T* __restrict__ col, int chunk_cols, int chunks,
                                                              int part_rows, int wp, int rsplit) {
  extern __shared__ float tile[];
  int b = blockIdx.x;
  // kernel rows [r_begin, r_end) of this block: tall kernels are split over blocks for parallelism
  const int rpart = b % rsplit;
  b /= rsplit;
  const int rper = (g.r + rsplit - 1) / rsplit;
  const int r_begin = rpart * rper, r_end = min(g.r, r_begin + rper);
  const int chunk = b % chunks;
  const int c = b / chunks;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // columns [j0, j1) = pixels from (n_first, oy_first, .) to (n_last, oy_last, .)
  const int P = (int)g.P;
  const int j0 = chunk * chunk_cols, j1 = (int)min((int64_t)j0 + chunk_cols, g.N);
  const int n_first = j0 / P, n_last = (j1 - 1) / P;
  const int oy_first = (j0 - n_first * P) / g.ow, oy_last = (j1 - 1 - n_last * P) / g.ow;
  const int nparts = n_last - n_first + 1;

  // Part i (image n_first+i) owns tile rows [i*part_rows, (i+1)*part_rows); its tile row 0 is input row
  // lo - ph + r_begin, lo = its first output row in the chunk.
  for (int idx = wave; idx < nparts * part_rows; idx += kThreads / 64) {
    const int i = idx / part_rows, ry = idx - i * part_rows;
    const int lo = i == 0 ? oy_first : 0, hi = i == nparts - 1 ? oy_last : g.oh - 1;
    if (ry >= hi - lo + r_end - r_begin) continue;
    const int ih = lo - g.ph + r_begin + ry;
    const bool row_ok = ih >= 0 && ih < g.h;
    const T* src = x + (((int64_t)(n_first + i) * g.c + c) * g.h + (row_ok ? ih : 0)) * g.w;
    for (int rx = lane; rx < wp; rx += 64) {
      const int iw = rx - g.pw;
      const bool ok = row_ok && iw >= 0 && iw < g.w;
      const float v = ld(src + (ok ? iw : 0));
      tile[idx * wp + rx] = ok ? v : 0.f;
    }
  }
  __syncthreads();

  // This thread's run of four consecutive columns (it may straddle an output row or an image).
  const int q0 = j0 + threadIdx.x * kVec;
  if (q0 >= j1) return;
  int base[kVec];
#pragma unroll
  for (int e = 0; e < kVec; ++e) {
    const int j = min(q0 + e, j1 - 1);
    const int n = j / P, p = j - n * P;
    const int oy = p / g.ow, ox = p - oy * g.ow;
    const int i = n - n_first;
    base[e] = (i * part_rows + oy - (i == 0 ? oy_first : 0)) * wp + ox;
  }
  T* dst = col + ((int64_t)(c * g.r + r_begin) * g.s) * g.N + q0;
  if (ALIGNED && q0 + kVec <= j1) {
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
        st(dst, tile[base[0] + off]);
        if (q0 + 1 < j1) st(dst + 1, tile[base[1] + off]);
        if (q0 + 2 < j1) st(dst + 2, tile[base[2] + off]);
        if (q0 + 3 < j1) st(dst + 3, tile[base[3] + off]);
        dst += g.N;
      }
  }
}

vcnn_status launch_im2col(const ConvGeom& g, int dtype, const void* x, void* col, hipStream_t st) {
  const int wp = g.w + 2 * g.pw;
  if (g.N > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "im2col: more than 2^31-1 patch-matrix columns");
  if (g.N == 0 || g.K == 0) return VCNN_OK;
  // Chunk: as many columns as one pass of the block covers, fewer (in steps of 32) while the staged tile
  // - per touched image the rows under the chunk plus the halo of the block's kernel rows - exceeds
  // 60 KB of LDS.  Tall kernels are split over blocks (fewer halo rows, and enough blocks in flight).
  const size_t row_bytes = (size_t)wp * sizeof(float);
  const int64_t max_rows = (int64_t)(60 * 1024 / row_bytes);  // tile rows that fit
  auto parts_of = [&](int cols) { return (int)((cols - 1) / g.P + 2); };           // images a chunk can touch
  auto rows_of = [&](int cols) { return (int)std::min<int64_t>(g.oh, (cols - 1) / g.ow + 2); };  // output rows of a part
  int chunk_cols = kThreads * kVec;
  while (chunk_cols > 32 && (int64_t)parts_of(chunk_cols) * rows_of(chunk_cols) > max_rows) chunk_cols -= 32;
  if ((int64_t)parts_of(chunk_cols) * rows_of(chunk_cols) > max_rows)
    return fail(VCNN_ERR_UNSUPPORTED, "im2col: padded input rows of %d floats do not fit the LDS tile", wp);
  const int parts = parts_of(chunk_cols), out_rows = rows_of(chunk_cols);
  const int rper_max = (int)(max_rows / parts) - out_rows + 1;  // >= 1
  const int chunks = (int)ceil_div(g.N, chunk_cols);
  int64_t rsplit = ceil_div(8192, (int64_t)g.c * chunks);
  if (rsplit < ceil_div(g.r, rper_max)) rsplit = ceil_div(g.r, rper_max);
  if (rsplit > g.r) rsplit = g.r;
  if (rsplit < 1) rsplit = 1;
  const int rper = (int)ceil_div(g.r, rsplit);
  rsplit = ceil_div(g.r, rper);  // no empty parts
  const int64_t blocks = (int64_t)g.c * chunks * rsplit;
  if (blocks > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "im2col: too many blocks for one launch");
  const int part_rows = out_rows + rper - 1;
  const size_t lds = (size_t)parts * part_rows * row_bytes;
  // 16-byte stores need the row pitch to be a multiple of four elements and an aligned matrix
  const dim3 grid((unsigned)blocks), block(kThreads);
  if (dtype == VCNN_BF16) {
    const bool aligned = g.N % kVec == 0 && group_aligned<bf16>(col);
    if (aligned)
      hipLaunchKernelGGL((im2col_f32_kernel<true, bf16>), grid, block, lds, st, g, (const bf16*)x, (bf16*)col,
                         chunk_cols, chunks, part_rows, wp, (int)rsplit);
    else
      hipLaunchKernelGGL((im2col_f32_kernel<false, bf16>), grid, block, lds, st, g, (const bf16*)x, (bf16*)col,
                         chunk_cols, chunks, part_rows, wp, (int)rsplit);
  } else {
    const bool aligned = g.N % kVec == 0 && group_aligned<float>(col);
    if (aligned)
      hipLaunchKernelGGL((im2col_f32_kernel<true, float>), grid, block, lds, st, g, (const float*)x, (float*)col,
                         chunk_cols, chunks, part_rows, wp, (int)rsplit);
    else
      hipLaunchKernelGGL((im2col_f32_kernel<false, float>), grid, block, lds, st, g, (const float*)x, (float*)col,
                         chunk_cols, chunks, part_rows, wp, (int)rsplit);
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
