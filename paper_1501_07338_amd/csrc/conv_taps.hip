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
// The products run in the generic matrix-core kernels of gemm.hip; this file holds the gather and the launch logic.
#include "common.h"
#include "elem.h"

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

bool conv_taps_applies(const ConvGeom& g) {
  // one map, enough channels for the contraction of the forward product, enough taps for its rows
  return g.k == 1 && g.c >= 32 && g.r * g.s >= 16 && g.r * g.s <= 1024 && g.r - 1 - g.ph >= 0 && g.s - 1 - g.pw >= 0 &&
         (int64_t)g.n * g.h * g.w <= 0x7fffffffLL;
}

size_t conv_taps_fwd_bytes(const ConvGeom& g) { return (size_t)g.n * g.r * g.s * g.h * g.w * sizeof(float); }

vcnn_status launch_conv_taps_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, const float* bias, void* y,
                                 int relu, float* z, hipStream_t st) {
  const int RS = g.r * g.s, HW = g.h * g.w;
  GemmArgs a{};
  a.A = w, a.B = x, a.C = z, a.bias = nullptr;
  a.in_dtype = dtype, a.out_dtype = VCNN_F32;
  a.M = RS, a.N = g.n * HW, a.K = g.c;
  a.a_si = 1, a.a_sk = RS;                                     // A(q, c) = w[c][q]
  a.b_sk = HW, a.b_sj = 1, a.b_P = HW, a.b_simg = (int64_t)g.c * HW;  // B(c, (n, pixel)) = x[n][c][pixel]
  a.c_si = HW, a.c_sj = 1, a.c_P = HW, a.c_simg = (int64_t)RS * HW;   // Z[n][q][pixel]
  if (vcnn_status s = launch_gemm_f32(a, st)) return s;
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
