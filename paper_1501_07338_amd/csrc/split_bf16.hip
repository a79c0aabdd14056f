// fp32 products of large layers as sums of bf16 products - a route taken only when asked for (VCNN_ALGO_SPLIT).
//
// The matrix cores of this chip multiply bfloat16 sixteen times as fast as float.  A float a is, exactly, the sum of
// three bfloat16 terms a1 + a2 + a3 (a1 = a rounded to bfloat16, a2 = the remainder rounded, a3 = what is left: 3 x 8
// significand bits).  A product a * b is then the sum of nine term products, each of them exact in float; the three
// smallest (a2 b3, a3 b2, a3 b3) lie below 2^-24 |a b|, the rounding a float product has anyway, and are left out.
// So the forward product (Eq. 1 / Eq. 2) and the kernel-gradient product of a layer are six bf16 products each,
// accumulated in float - smallest terms first, in a fixed order - through the bf16 kernels of the bf16 variant:
//     y  = sum over (i, j) in {(3,1), (1,3), (2,2), (2,1), (1,2), (1,1)} of  w_j (*) x_i
//     dw = the same sum of  dy_j (x) x_i
// The result carries an error of the size of float arithmetic (the tests hold it to the float tolerance), for six
// passes of a kernel that is an order of magnitude faster than the float one.
#include <algorithm>

#include "common.h"
#include "elem.h"

namespace vcnn {

static constexpr int kThreads = 256;

// p1 + p2 + p3 = src exactly (up to underflow of the last term)
__global__ __launch_bounds__(kThreads) void split3_kernel(const float* __restrict__ src, bf16* __restrict__ p1,
                                                          bf16* __restrict__ p2, bf16* __restrict__ p3, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= count) return;
  const float a = src[i];
  const uint16_t b1 = f32_to_bf16_bits(a);
  const float r1 = a - bf16_bits_to_f32(b1);
  const uint16_t b2 = f32_to_bf16_bits(r1);
  const float r2 = r1 - bf16_bits_to_f32(b2);
  p1[i].bits = b1, p2[i].bits = b2, p3[i].bits = f32_to_bf16_bits(r2);
}

static vcnn_status split3(const float* src, void* base, size_t part_bytes, int64_t count, hipStream_t st) {
  bf16* p1 = (bf16*)base;
  bf16* p2 = (bf16*)((char*)base + part_bytes);
  bf16* p3 = (bf16*)((char*)base + 2 * part_bytes);
  hipLaunchKernelGGL(split3_kernel, dim3((unsigned)ceil_div(count, kThreads)), dim3(kThreads), 0, st, src, p1, p2, p3, count);
  return check_launch("split3");
}

static inline size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// the six term pairs, smallest products first: {term of the first operand, term of the second}
static constexpr int kPairs[6][2] = {{2, 0}, {0, 2}, {1, 1}, {1, 0}, {0, 1}, {0, 0}};

bool conv_split_plan(const ConvGeom& g, int pass, SplitPlan* p) {
  if ((int64_t)g.n * g.c * g.h * g.w > 0x7fffffff00LL || g.M * g.N > 0x7fffffff00LL) return false;
  p->part_x_bytes = align256((size_t)g.n * g.c * g.h * g.w * 2);
  p->part_w_bytes = align256((size_t)g.M * g.K * 2);
  p->part_dy_bytes = align256((size_t)g.M * g.N * 2);
  if (pass == VCNN_PASS_FWD) {
    // many maps: the six term products inside one kernel; else six passes of the bfloat16 kernel
    if (g.k <= 4 || !(conv_halo_bf16_plan(g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, &p->fwd, 3) ||
                      conv_halo_bf16_plan(g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, &p->fwd)))
      return false;
    p->inner_bytes = 3 * (p->fwd.x8_bytes + p->fwd.wf_bytes);  // every term of both operands re-laid once
    p->workspace_bytes = 3 * p->part_x_bytes + 3 * p->part_w_bytes + p->inner_bytes;
    return true;
  }
  if (pass == VCNN_PASS_BWD_FILTER) {
    if (g.k <= 4 || g.c <= 4 || !(filter_grad_bf16_plan(g, &p->filter, 3) || filter_grad_bf16_plan(g, &p->filter))) return false;
    const size_t slices = std::max(p->filter.partial_bytes, (size_t)g.M * g.K * sizeof(float));
    p->inner_bytes = 3 * (p->filter.x8n_bytes + p->filter.dyf_bytes) + align256(slices);
    p->workspace_bytes = 3 * p->part_x_bytes + 3 * p->part_dy_bytes + p->inner_bytes;
    return true;
  }
  return false;
}

vcnn_status launch_conv_split_fwd(const SplitPlan& p, const ConvGeom& g, const float* x, const float* w, const float* bias,
                                  float* y, int relu, void* workspace, hipStream_t st) {
  char* xs = (char*)workspace;
  char* ws = xs + 3 * p.part_x_bytes;
  char* x8s = ws + 3 * p.part_w_bytes;       // three channel-interleaved terms of x
  char* wfs = x8s + 3 * p.fwd.x8_bytes;      // three fragment-ordered terms of w
  if (vcnn_status e = split3(x, xs, p.part_x_bytes, (int64_t)g.n * g.c * g.h * g.w, st)) return e;
  if (vcnn_status e = split3(w, ws, p.part_w_bytes, g.M * g.K, st)) return e;
  if (p.fwd.terms == 3)
    return launch_conv_halo_bf16_terms(p.fwd, g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, xs, p.part_x_bytes, ws,
                                       p.part_w_bytes, g.K, (int64_t)g.r * g.s, bias, y, relu, x8s, wfs, st);
  bool x_done[3] = {false, false, false}, w_done[3] = {false, false, false};
  for (int t = 0; t < 6; ++t) {
    const int i = kPairs[t][0], j = kPairs[t][1];
    const void* xi = x_done[i] ? nullptr : xs + i * p.part_x_bytes;  // re-laid on first use only
    const void* wj = w_done[j] ? nullptr : ws + j * p.part_w_bytes;
    x_done[i] = w_done[j] = true;
    const bool first = t == 0, last = t == 5;
    if (vcnn_status e = launch_conv_halo_bf16_prepared(p.fwd, g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, xi, wj, g.K,
                                                       (int64_t)g.r * g.s, 0, first ? bias : nullptr, nullptr,
                                                       last ? relu : 0, x8s + i * p.fwd.x8_bytes, wfs + j * p.fwd.wf_bytes, st,
                                                       y, first ? 0 : 1))
      return e;
  }
  return VCNN_OK;
}

vcnn_status launch_conv_split_filter(const SplitPlan& p, const ConvGeom& g, const float* x, const float* dy, float* dw,
                                     void* workspace, hipStream_t st) {
  char* xs = (char*)workspace;
  char* ds = xs + 3 * p.part_x_bytes;
  char* x8s = ds + 3 * p.part_dy_bytes;           // three image-interleaved terms of x
  char* dfs = x8s + 3 * p.filter.x8n_bytes;       // three fragment-ordered terms of dy
  float* slices = (float*)(dfs + 3 * p.filter.dyf_bytes);
  if (vcnn_status e = split3(x, xs, p.part_x_bytes, (int64_t)g.n * g.c * g.h * g.w, st)) return e;
  if (vcnn_status e = split3(dy, ds, p.part_dy_bytes, g.M * g.N, st)) return e;
  if (p.filter.terms == 3)
    return launch_filter_grad_bf16_terms(p.filter, g, xs, p.part_x_bytes, ds, p.part_dy_bytes, dw, x8s, dfs, slices, st);
  bool x_done[3] = {false, false, false}, d_done[3] = {false, false, false};
  for (int t = 0; t < 6; ++t) {
    const int i = kPairs[t][0], j = kPairs[t][1];
    const void* xi = x_done[i] ? nullptr : xs + i * p.part_x_bytes;  // re-laid on first use only
    const void* dj = d_done[j] ? nullptr : ds + j * p.part_dy_bytes;
    x_done[i] = d_done[j] = true;
    if (vcnn_status e = launch_filter_grad_bf16_prepared(p.filter, g, xi, dj, dw, x8s + i * p.filter.x8n_bytes,
                                                         dfs + j * p.filter.dyf_bytes, slices, st, t == 0 ? 0 : 1))
      return e;
  }
  return VCNN_OK;
}

}  // namespace vcnn
