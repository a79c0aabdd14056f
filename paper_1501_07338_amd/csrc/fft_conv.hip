// Forward pass of layers with one-dimensional kernels (r x 1 or 1 x s) through the Fourier domain - the "FFT
// speedup" the paper's related-work paragraph sets beside its own unrolling.  A comparison route, taken only
// when asked for (VCNN_ALGO_FFT): the vectorized path is the unroll + matrix product.
//
// Along the kernel's axis the layer is, for every line q = (sample, position on the other axis),
//     y[k][q][o] = bias[k] + sum_c sum_t w[k][c][t] * x[c][q][o + t - pad],     o = 0 .. out_len - 1,
// a correlation of zero-extended lines.  With L a power of two >= pad + len (so nothing wraps around),
//     Y^[k][q][f] = sum_c conj(W^[k][c][f]) * X^[c][q][f],   X^ = DFT_L(x shifted right by pad), W^ = DFT_L(w),
// and y = the first out_len entries of the inverse transform.  Four kernels: lines -> X^ (half spectrum, the
// lines being real), kernels -> conj(W^), the contraction over the input channels frequency by frequency, and the
// inverse transform with bias and sigma.  Transforms are radix-2 Stockham autosort FFTs in LDS, one butterfly per
// thread and stage, twiddle factors from a table computed with sincospi.
#include <algorithm>

#include "common.h"
#include "elem.h"

namespace vcnn {

static constexpr int kThreads = 256;

struct FftArgs {
  const void* x;      // [n][c][h][w], element type T
  const void* wgt;    // [k][c][taps]
  const float* bias;  // [k] or null
  void* y;            // [n][k][oh][ow]
  float2* xf;         // [c][Q][LP]
  float2* wf;         // [k][c][LP]   conjugated
  float2* yf;         // [k][Q][LP]
  int n, c, h, w, k, taps, pad, oh, ow;
  int along_w;        // 1: 1 x s kernels (lines are image rows), 0: r x 1 kernels (lines are image columns)
  int len, out_len;   // line length in / out along the kernel's axis
  int other;          // positions on the other axis (lines per sample and channel)
  int Q;              // n * other
  int L, logL, LP;    // transform length, its log2, L/2 + 1
  int relu;
};

__device__ __forceinline__ float2 cmul(float2 a, float2 b) { return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }

// In-place (ping-pong) Stockham radix-2 transform of `lines` sequences of length L held in buf[0] (layout
// [line][L]); returns the buffer index that holds the result.  All kThreads threads take part; SIGN = -1 forward,
// +1 inverse (unscaled).  tw[m] = exp(-2 pi i m / L), m < L/2.
template <int SIGN>
__device__ __forceinline__ int fft_lds(float2* buf0, float2* buf1, const float2* tw, int lines, int L, int logL, int tid) {
  float2* in = buf0;
  float2* out = buf1;
  const int half = L >> 1;
  const int work = lines * half;  // butterflies per stage
  for (int s = 0; s < logL; ++s) {
    const int p = 1 << s;
    for (int e = tid; e < work; e += kThreads) {
      const int line = e / half, j = e - line * half;
      const int kk = j & (p - 1);
      float2 t = tw[kk * (half >> s)];  // exp(-i pi kk / p)
      if (SIGN > 0) t.y = -t.y;
      const float2 u = in[line * L + j];
      const float2 v = cmul(in[line * L + j + half], t);
      const int j0 = ((j - kk) << 1) + kk;
      out[line * L + j0] = make_float2(u.x + v.x, u.y + v.y);
      out[line * L + j0 + p] = make_float2(u.x - v.x, u.y - v.y);
    }
    __syncthreads();
    float2* tmp = in;
    in = out;
    out = tmp;
  }
  return (logL & 1) ? 1 : 0;
}

__device__ __forceinline__ void fill_twiddles(float2* tw, int L, int tid) {
  for (int m = tid; m < L / 2; m += kThreads) {
    float s, c;
    sincospif(-2.0f * (float)m / (float)L, &s, &c);
    tw[m] = make_float2(c, s);
  }
}

// address of element t of line (n, ch, o) of a [n][C][h][w] tensor
__device__ __forceinline__ int64_t line_elem(const FftArgs& a, int C, int H, int W, int n, int ch, int o, int t) {
  return a.along_w ? (((int64_t)n * C + ch) * H + o) * W + t : (((int64_t)n * C + ch) * H + t) * W + o;
}

// Lines of the input -> half spectra.  A block transforms SB lines of one channel: consecutive positions on the
// other axis (for column lines those are neighbouring addresses, so the loads coalesce across lines).
template <typename T>
__global__ __launch_bounds__(kThreads) void fft_lines_kernel(FftArgs a, int SB) {
  extern __shared__ float4 smem4[];
  float2* tw = reinterpret_cast<float2*>(smem4);
  float2* b0 = tw + a.L / 2;
  float2* b1 = b0 + SB * a.L;
  const int tid = threadIdx.x;
  const int groups = (a.other + SB - 1) / SB;
  int g = blockIdx.x;
  const int og = g % groups;
  g /= groups;
  const int ch = g % a.c, n = g / a.c;
  const int o0 = og * SB;
  const T* x = static_cast<const T*>(a.x);
  fill_twiddles(tw, a.L, tid);
  // stage: element t of line l sits at position t + pad (zero elsewhere)
  for (int e = tid; e < SB * a.L; e += kThreads) {
    int l, pos;
    if (a.along_w) l = e / a.L, pos = e - l * a.L;
    else pos = e / SB, l = e - pos * SB;
    const int t = pos - a.pad;
    float v = 0.f;
    if (o0 + l < a.other && t >= 0 && t < a.len) v = ld(x + line_elem(a, a.c, a.h, a.w, n, ch, o0 + l, t));
    b0[l * a.L + pos] = make_float2(v, 0.f);
  }
  __syncthreads();
  const int res = fft_lds<-1>(b0, b1, tw, SB, a.L, a.logL, tid);
  const float2* r = res ? b1 : b0;
  for (int e = tid; e < SB * a.LP; e += kThreads) {
    const int l = e / a.LP, f = e - l * a.LP;
    if (o0 + l < a.other) a.xf[((int64_t)ch * a.Q + (int64_t)n * a.other + o0 + l) * a.LP + f] = r[l * a.L + f];
  }
}

// Kernels -> conjugated half spectra wf[k][c][f].
template <typename T>
__global__ __launch_bounds__(kThreads) void fft_kernels_kernel(FftArgs a, int SB) {
  extern __shared__ float4 smem4[];
  float2* tw = reinterpret_cast<float2*>(smem4);
  float2* b0 = tw + a.L / 2;
  float2* b1 = b0 + SB * a.L;
  const int tid = threadIdx.x;
  const int total = a.k * a.c;
  const int l0 = blockIdx.x * SB;
  const T* w = static_cast<const T*>(a.wgt);
  fill_twiddles(tw, a.L, tid);
  for (int e = tid; e < SB * a.L; e += kThreads) {
    const int l = e / a.L, pos = e - l * a.L;
    float v = 0.f;
    if (l0 + l < total && pos < a.taps) v = ld(w + (int64_t)(l0 + l) * a.taps + pos);
    b0[e] = make_float2(v, 0.f);
  }
  __syncthreads();
  const int res = fft_lds<-1>(b0, b1, tw, SB, a.L, a.logL, tid);
  const float2* r = res ? b1 : b0;
  for (int e = tid; e < SB * a.LP; e += kThreads) {
    const int l = e / a.LP, f = e - l * a.LP;
    if (l0 + l < total) {
      const float2 v = r[l * a.L + f];
      a.wf[(int64_t)(l0 + l) * a.LP + f] = make_float2(v.x, -v.y);
    }
  }
}

// yf[k][q][f] = sum_c wf[k][c][f] * xf[c][q][f].  A block owns FT frequencies x 64 lines for KB output maps at a
// time; the kernels' spectra for those frequencies sit in LDS, every thread keeps KB complex sums.
static constexpr int kFT = 4, kKB = 16;
__global__ __launch_bounds__(kThreads) void freq_contract_kernel(FftArgs a) {
  extern __shared__ float4 smem4[];
  float2* ws = reinterpret_cast<float2*>(smem4);  // [KB][c][FT]
  const int tid = threadIdx.x;
  const int fl = tid & (kFT - 1), ql = tid / kFT;
  const int ftiles = (a.LP + kFT - 1) / kFT;
  const int ft = blockIdx.x % ftiles, qt = blockIdx.x / ftiles;
  const int f = ft * kFT + fl, q = qt * (kThreads / kFT) + ql;
  const bool ok = f < a.LP && q < a.Q;
  const int fc = min(f, a.LP - 1), qc = min(q, a.Q - 1);
  for (int k0 = 0; k0 < a.k; k0 += kKB) {
    const int kb = min(kKB, a.k - k0);
    __syncthreads();
    for (int e = tid; e < kb * a.c * kFT; e += kThreads) {
      const int ff = e % kFT, kc = e / kFT;  // kc = kl * c + ch
      const int fg = min(ft * kFT + ff, a.LP - 1);
      ws[e] = a.wf[((int64_t)k0 * a.c + kc) * a.LP + fg];
    }
    __syncthreads();
    float2 acc[kKB];
#pragma unroll
    for (int kl = 0; kl < kKB; ++kl) acc[kl] = make_float2(0.f, 0.f);
    for (int ch = 0; ch < a.c; ++ch) {
      const float2 xv = a.xf[((int64_t)ch * a.Q + qc) * a.LP + fc];
#pragma unroll
      for (int kl = 0; kl < kKB; ++kl)
        if (kl < kb) {
          const float2 wv = ws[(kl * a.c + ch) * kFT + fl];
          acc[kl].x += wv.x * xv.x - wv.y * xv.y;
          acc[kl].y += wv.x * xv.y + wv.y * xv.x;
        }
    }
    if (ok) {
#pragma unroll
      for (int kl = 0; kl < kKB; ++kl)
        if (kl < kb) a.yf[((int64_t)(k0 + kl) * a.Q + q) * a.LP + f] = acc[kl];
    }
  }
}

// Half spectra of the result -> lines of y: Hermitian extension, inverse transform, scale 1/L, bias, sigma.
template <typename T>
__global__ __launch_bounds__(kThreads) void ifft_lines_kernel(FftArgs a, int SB) {
  extern __shared__ float4 smem4[];
  float2* tw = reinterpret_cast<float2*>(smem4);
  float2* b0 = tw + a.L / 2;
  float2* b1 = b0 + SB * a.L;
  const int tid = threadIdx.x;
  const int groups = (a.other + SB - 1) / SB;
  int g = blockIdx.x;
  const int og = g % groups;
  g /= groups;
  const int km = g % a.k, n = g / a.k;
  const int o0 = og * SB;
  fill_twiddles(tw, a.L, tid);
  for (int e = tid; e < SB * a.L; e += kThreads) {
    const int l = e / a.L, f = e - l * a.L;
    float2 v = make_float2(0.f, 0.f);
    if (o0 + l < a.other) {
      const float2* src = a.yf + ((int64_t)km * a.Q + (int64_t)n * a.other + o0 + l) * a.LP;
      if (f < a.LP) v = src[f];
      else {
        v = src[a.L - f];
        v.y = -v.y;
      }
    }
    b0[e] = v;
  }
  __syncthreads();
  const int res = fft_lds<1>(b0, b1, tw, SB, a.L, a.logL, tid);
  const float2* r = res ? b1 : b0;
  T* y = static_cast<T*>(a.y);
  const float scale = 1.f / (float)a.L;
  const float bv = a.bias ? a.bias[km] : 0.f;
  for (int e = tid; e < SB * a.out_len; e += kThreads) {
    int l, t;
    if (a.along_w) l = e / a.out_len, t = e - l * a.out_len;
    else t = e / SB, l = e - t * SB;
    if (o0 + l >= a.other) continue;
    float v = r[l * a.L + t].x * scale + bv;
    if (a.relu) v = fmaxf(v, 0.f);
    st(y + line_elem(a, a.k, a.oh, a.ow, n, km, o0 + l, t), v);
  }
}

bool conv_fft_plan(const ConvGeom& g, FftPlan* p) {
  const bool row_kernel = g.r == 1 && g.ph == 0, col_kernel = g.s == 1 && g.pw == 0;
  if (!row_kernel && !col_kernel) return false;
  if (row_kernel && col_kernel) return false;  // 1 x 1: nothing to transform
  p->along_w = row_kernel ? 1 : 0;
  p->len = row_kernel ? g.w : g.h;
  p->taps = row_kernel ? g.s : g.r;
  p->pad = row_kernel ? g.pw : g.ph;
  p->out_len = row_kernel ? g.ow : g.oh;
  p->other = row_kernel ? g.h : g.w;
  if (p->taps < 8) return false;  // short kernels gain nothing from the transform
  const int need = p->len + p->pad;  // the shifted line; outputs o < out_len read positions < len + pad: no wrap-around
  int L = 32, logL = 5;
  while (L < need || L < p->taps) L <<= 1, ++logL;
  if (L > 1024) return false;
  p->L = L, p->logL = logL, p->LP = L / 2 + 1;
  const int64_t Q = (int64_t)g.n * p->other;
  if (Q * p->LP * std::max(g.c, g.k) > 0x7fffffffLL) return false;
  p->Q = (int)Q;
  // lines per block; column lines take more of them, neighbouring lines being neighbouring addresses
  p->sb = p->along_w ? std::max(1, 1024 / L) : std::max(1, 2048 / L);
  p->xf_bytes = ((size_t)g.c * Q * p->LP * sizeof(float2) + 255) & ~(size_t)255;
  p->wf_bytes = ((size_t)g.k * g.c * p->LP * sizeof(float2) + 255) & ~(size_t)255;
  p->yf_bytes = ((size_t)g.k * Q * p->LP * sizeof(float2) + 255) & ~(size_t)255;
  return true;
}

vcnn_status launch_conv_fft(const FftPlan& p, int dtype, const ConvGeom& g, const void* x, const void* w, const float* bias,
                            void* y, int relu, void* workspace, hipStream_t st) {
  FftArgs a{};
  a.x = x, a.wgt = w, a.bias = bias, a.y = y;
  a.xf = (float2*)workspace;
  a.wf = (float2*)((char*)workspace + p.xf_bytes);
  a.yf = (float2*)((char*)workspace + p.xf_bytes + p.wf_bytes);
  a.n = g.n, a.c = g.c, a.h = g.h, a.w = g.w, a.k = g.k, a.taps = p.taps, a.pad = p.pad, a.oh = g.oh, a.ow = g.ow;
  a.along_w = p.along_w, a.len = p.len, a.out_len = p.out_len, a.other = p.other, a.Q = p.Q;
  a.L = p.L, a.logL = p.logL, a.LP = p.LP, a.relu = relu;
  const int SB = p.sb;
  const size_t lds = ((size_t)p.L / 2 + 2 * (size_t)SB * p.L) * sizeof(float2);
  const dim3 block(kThreads);
  const int groups = (p.other + SB - 1) / SB;
  const bool bf = dtype == VCNN_BF16;
  {
    const dim3 grid((unsigned)((int64_t)g.n * g.c * groups));
    if (bf) hipLaunchKernelGGL(fft_lines_kernel<bf16>, grid, block, lds, st, a, SB);
    else hipLaunchKernelGGL(fft_lines_kernel<float>, grid, block, lds, st, a, SB);
    if (vcnn_status s = check_launch("fft_lines")) return s;
  }
  {
    const dim3 grid((unsigned)ceil_div((int64_t)g.k * g.c, SB));
    if (bf) hipLaunchKernelGGL(fft_kernels_kernel<bf16>, grid, block, lds, st, a, SB);
    else hipLaunchKernelGGL(fft_kernels_kernel<float>, grid, block, lds, st, a, SB);
    if (vcnn_status s = check_launch("fft_kernels")) return s;
  }
  {
    const int ftiles = (p.LP + kFT - 1) / kFT;
    const dim3 grid((unsigned)((int64_t)ftiles * ceil_div(p.Q, kThreads / kFT)));
    const size_t wlds = (size_t)kKB * g.c * kFT * sizeof(float2);
    if (wlds > 64 * 1024) return fail(VCNN_ERR_UNSUPPORTED, "conv_fft: %d input channels are too many for the contraction kernel", g.c);
    hipLaunchKernelGGL(freq_contract_kernel, grid, block, wlds, st, a);
    if (vcnn_status s = check_launch("freq_contract")) return s;
  }
  {
    const dim3 grid((unsigned)((int64_t)g.n * g.k * groups));
    if (bf) hipLaunchKernelGGL(ifft_lines_kernel<bf16>, grid, block, lds, st, a, SB);
    else hipLaunchKernelGGL(ifft_lines_kernel<float>, grid, block, lds, st, a, SB);
  }
  return check_launch("ifft_lines");
}

}  // namespace vcnn
