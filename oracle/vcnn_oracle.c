/*
 * fp64 CPU oracle for the vectorized CNN layer path of Ren & Xu, "On Vectorization of Deep
 * Convolutional Neural Networks for Vision Tasks" (AAAI 2015).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file; it exists so the HIP
 * kernels can be checked against the plain definitions.  It shares no code with them.
 *
 * The unroll-then-multiply formulation of the paper (Eq. 2 and Eq. 4) is an exact re-association of
 * the direct sums, so the oracle is the direct sums: literal nested loops in double precision, no
 * unrolled patch matrix, no blocked matrix product.  OpenMP is used only over the outermost
 * independent output loops; every output element is produced by one thread in a fixed order.
 *
 * Layouts (dense, contiguous): activations [N][C][H][W]; conv weights [K][C][R][S]; fc weights
 * [O][I]; the unrolled patch matrix is [C*R*S][N*OH*OW] with s fastest in a row index and ow fastest
 * in a column index.
 *
 * Reading of the paper's "*" (Eq. 1): cross-correlation (no kernel flip), which is what stacking
 * patches as columns and kernels as rows ("Matlab Practice" paragraph, Fig. 2) computes.
 * Padding is zero extension followed by the valid operation (the paper considers the valid region).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

typedef int64_t i64;

static inline i64 out_dim(i64 in, i64 k, i64 pad, i64 stride) { return (in + 2 * pad - k) / stride + 1; }

/* Eq. 1: y[n,k,oh,ow] = sigma(b[k] + sum_{c,r,s} w[k,c,r,s] * xpad[n,c,oh*sh+r-ph,ow*sw+s-pw]). */
void oracle_conv_fwd(const double *x, const double *w, const double *b, double *y, int N, int C, int H,
                     int W, int K, int R, int S, int ph, int pw, int sh, int sw, int relu) {
  const i64 OH = out_dim(H, R, ph, sh), OW = out_dim(W, S, pw, sw);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (i64 n = 0; n < N; ++n)
    for (i64 k = 0; k < K; ++k)
      for (i64 oh = 0; oh < OH; ++oh)
        for (i64 ow = 0; ow < OW; ++ow) {
          double acc = b ? b[k] : 0.0;
          for (i64 c = 0; c < C; ++c)
            for (i64 r = 0; r < R; ++r) {
              const i64 ih = oh * sh + r - ph;
              if (ih < 0 || ih >= H) continue; /* zero padding contributes nothing */
              for (i64 s = 0; s < S; ++s) {
                const i64 iw = ow * sw + s - pw;
                if (iw < 0 || iw >= W) continue;
                acc += w[((k * C + c) * R + r) * S + s] * x[((n * C + c) * H + ih) * W + iw];
              }
            }
          if (relu && acc < 0.0) acc = 0.0;
          y[((n * K + k) * OH + oh) * OW + ow] = acc;
        }
}

/* Derivative of Eq. 1's linear part w.r.t. the kernels:
 * dw[k,c,r,s] = sum_{n,oh,ow} dy[n,k,oh,ow] * xpad[n,c,oh*sh+r-ph,ow*sw+s-pw];  db[k] = sum dy[:,k,:,:]. */
void oracle_conv_bwd_filter(const double *x, const double *dy, double *dw, double *db, int N, int C, int H,
                            int W, int K, int R, int S, int ph, int pw, int sh, int sw) {
  const i64 OH = out_dim(H, R, ph, sh), OW = out_dim(W, S, pw, sw);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (i64 k = 0; k < K; ++k)
    for (i64 c = 0; c < C; ++c)
      for (i64 r = 0; r < R; ++r)
        for (i64 s = 0; s < S; ++s) {
          double acc = 0.0;
          for (i64 n = 0; n < N; ++n)
            for (i64 oh = 0; oh < OH; ++oh) {
              const i64 ih = oh * sh + r - ph;
              if (ih < 0 || ih >= H) continue;
              for (i64 ow = 0; ow < OW; ++ow) {
                const i64 iw = ow * sw + s - pw;
                if (iw < 0 || iw >= W) continue;
                acc += dy[((n * K + k) * OH + oh) * OW + ow] * x[((n * C + c) * H + ih) * W + iw];
              }
            }
          dw[((k * C + c) * R + r) * S + s] = acc;
        }
  if (db) {
    for (i64 k = 0; k < K; ++k) {
      double acc = 0.0;
      for (i64 n = 0; n < N; ++n)
        for (i64 p = 0; p < OH * OW; ++p) acc += dy[(n * K + k) * OH * OW + p];
      db[k] = acc;
    }
  }
}

/* The many-to-one inverse of the unroll, composed with the kernel product (back-propagation
 * paragraph of the "Vectorizing Convolution" section): every input pixel collects the gradient of
 * every output it fed.  dx[n,c,h,w] = sum_{k,r,s : oh*sh+r-ph==h, ow*sw+s-pw==w} w[k,c,r,s]*dy[n,k,oh,ow]. */
void oracle_conv_bwd_data(const double *w, const double *dy, double *dx, int N, int C, int H, int W, int K,
                          int R, int S, int ph, int pw, int sh, int sw) {
  const i64 OH = out_dim(H, R, ph, sh), OW = out_dim(W, S, pw, sw);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (i64 n = 0; n < N; ++n)
    for (i64 c = 0; c < C; ++c)
      for (i64 h = 0; h < H; ++h)
        for (i64 wi = 0; wi < W; ++wi) {
          double acc = 0.0;
          for (i64 k = 0; k < K; ++k)
            for (i64 r = 0; r < R; ++r) {
              const i64 th = h + ph - r;
              if (th < 0 || th % sh != 0) continue;
              const i64 oh = th / sh;
              if (oh >= OH) continue;
              for (i64 s = 0; s < S; ++s) {
                const i64 tw = wi + pw - s;
                if (tw < 0 || tw % sw != 0) continue;
                const i64 ow = tw / sw;
                if (ow >= OW) continue;
                acc += w[((k * C + c) * R + r) * S + s] * dy[((n * K + k) * OH + oh) * OW + ow];
              }
            }
          dx[((n * C + c) * H + h) * W + wi] = acc;
        }
}

/* phi_c of Eq. 2 / Eq. 4: one column per output position of every sample, samples side by side. */
void oracle_im2col(const double *x, double *col, int N, int C, int H, int W, int R, int S, int ph, int pw,
                   int sh, int sw) {
  const i64 OH = out_dim(H, R, ph, sh), OW = out_dim(W, S, pw, sw);
  const i64 NC = (i64)N * OH * OW;
  for (i64 c = 0; c < C; ++c)
    for (i64 r = 0; r < R; ++r)
      for (i64 s = 0; s < S; ++s) {
        const i64 row = (c * R + r) * S + s;
        for (i64 n = 0; n < N; ++n)
          for (i64 oh = 0; oh < OH; ++oh)
            for (i64 ow = 0; ow < OW; ++ow) {
              const i64 ih = oh * sh + r - ph, iw = ow * sw + s - pw;
              double v = 0.0;
              if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = x[((n * C + c) * H + ih) * W + iw];
              col[row * NC + (n * OH + oh) * OW + ow] = v;
            }
      }
}

/* phi_c^{-1}: the many-to-one map; entries that were copies of one pixel are summed (scatter form). */
void oracle_col2im(const double *col, double *dx, int N, int C, int H, int W, int R, int S, int ph, int pw,
                   int sh, int sw) {
  const i64 OH = out_dim(H, R, ph, sh), OW = out_dim(W, S, pw, sw);
  const i64 NC = (i64)N * OH * OW;
  for (i64 i = 0; i < (i64)N * C * H * W; ++i) dx[i] = 0.0;
  for (i64 c = 0; c < C; ++c)
    for (i64 r = 0; r < R; ++r)
      for (i64 s = 0; s < S; ++s) {
        const i64 row = (c * R + r) * S + s;
        for (i64 n = 0; n < N; ++n)
          for (i64 oh = 0; oh < OH; ++oh)
            for (i64 ow = 0; ow < OW; ++ow) {
              const i64 ih = oh * sh + r - ph, iw = ow * sw + s - pw;
              if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                dx[((n * C + c) * H + ih) * W + iw] += col[row * NC + (n * OH + oh) * OW + ow];
            }
      }
}

/* phi_p with the max operation (Eq. 3 without bias and sigma): windows scanned in row-major order
 * with a strict '>' update, so among equal maxima the lowest flat index h*W+w wins.  No padding;
 * output size floor((H-win)/stride)+1. */
void oracle_maxpool_fwd(const double *x, double *y, int32_t *argmax, int N, int C, int H, int W, int wh,
                        int ww, int sh, int sw) {
  const i64 OH = (H - wh) / sh + 1, OW = (W - ww) / sw + 1;
#pragma omp parallel for schedule(static)
  for (i64 nc = 0; nc < (i64)N * C; ++nc) {
    const double *xp = x + nc * H * W;
    for (i64 oh = 0; oh < OH; ++oh)
      for (i64 ow = 0; ow < OW; ++ow) {
        double best = 0.0;
        int32_t bi = -1;
        for (i64 i = 0; i < wh; ++i)
          for (i64 j = 0; j < ww; ++j) {
            const i64 h = oh * sh + i, w = ow * sw + j;
            const double v = xp[h * W + w];
            if (bi < 0 || v > best) {
              best = v;
              bi = (int32_t)(h * W + w);
            }
          }
        y[(nc * OH + oh) * OW + ow] = best;
        argmax[(nc * OH + oh) * OW + ow] = bi;
      }
  }
}

/* Exact sub-gradient of max pooling: each output's gradient goes to the recorded position;
 * overlapping windows that chose the same position add up. */
void oracle_maxpool_bwd(const double *dy, const int32_t *argmax, double *dx, int N, int C, int H, int W,
                        int OH, int OW) {
  for (i64 i = 0; i < (i64)N * C * H * W; ++i) dx[i] = 0.0;
  for (i64 nc = 0; nc < (i64)N * C; ++nc)
    for (i64 p = 0; p < (i64)OH * OW; ++p) dx[nc * H * W + argmax[nc * OH * OW + p]] += dy[nc * OH * OW + p];
}

/* sigma = ReLU: y = max(x, 0); derivative taken as 0 at x <= 0. */
void oracle_relu_fwd(const double *x, double *y, i64 count) {
  for (i64 i = 0; i < count; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}
void oracle_relu_bwd(const double *x, const double *dy, double *dx, i64 count) {
  for (i64 i = 0; i < count; ++i) dx[i] = x[i] > 0.0 ? dy[i] : 0.0;
}

/* The other nonlinear functions Eq. 1 names for sigma: hyperbolic tangent and the logistic sigmoid.  The
 * derivatives are written in terms of the forward OUTPUT y: tanh' = 1 - y^2, sigmoid' = y (1 - y). */
void oracle_tanh_fwd(const double *x, double *y, i64 count) {
  for (i64 i = 0; i < count; ++i) y[i] = tanh(x[i]);
}
void oracle_tanh_bwd(const double *y, const double *dy, double *dx, i64 count) {
  for (i64 i = 0; i < count; ++i) dx[i] = dy[i] * (1.0 - y[i] * y[i]);
}
void oracle_sigmoid_fwd(const double *x, double *y, i64 count) {
  for (i64 i = 0; i < count; ++i) y[i] = 1.0 / (1.0 + exp(-x[i]));
}
void oracle_sigmoid_bwd(const double *y, const double *dy, double *dx, i64 count) {
  for (i64 i = 0; i < count; ++i) dx[i] = dy[i] * y[i] * (1.0 - y[i]);
}

/* phi_p with the average operation ("Vectorizing Pooling"): mean of each window; same window geometry as
 * max pooling (no padding, output floor((H-win)/stride)+1). */
void oracle_avgpool_fwd(const double *x, double *y, int N, int C, int H, int W, int wh, int ww, int sh, int sw) {
  const i64 OH = (H - wh) / sh + 1, OW = (W - ww) / sw + 1;
#pragma omp parallel for schedule(static)
  for (i64 nc = 0; nc < (i64)N * C; ++nc) {
    const double *xp = x + nc * H * W;
    for (i64 oh = 0; oh < OH; ++oh)
      for (i64 ow = 0; ow < OW; ++ow) {
        double sum = 0.0;
        for (i64 i = 0; i < wh; ++i)
          for (i64 j = 0; j < ww; ++j) sum += xp[(oh * sh + i) * W + ow * sw + j];
        y[(nc * OH + oh) * OW + ow] = sum / (double)(wh * ww);
      }
  }
}

/* Exact gradient of average pooling (the transpose of the linear map above): every position of a window
 * receives the window's gradient divided by the window size; overlapping windows add up.  For windows
 * that tile the plane (stride = window) this is the nearest-neighbour upscaling of dy the paper uses,
 * scaled by 1/(wh*ww). */
void oracle_avgpool_bwd(const double *dy, double *dx, int N, int C, int H, int W, int wh, int ww, int sh, int sw) {
  const i64 OH = (H - wh) / sh + 1, OW = (W - ww) / sw + 1;
  for (i64 i = 0; i < (i64)N * C * H * W; ++i) dx[i] = 0.0;
  for (i64 nc = 0; nc < (i64)N * C; ++nc)
    for (i64 oh = 0; oh < OH; ++oh)
      for (i64 ow = 0; ow < OW; ++ow) {
        const double g = dy[(nc * OH + oh) * OW + ow] / (double)(wh * ww);
        for (i64 i = 0; i < wh; ++i)
          for (i64 j = 0; j < ww; ++j) dx[nc * H * W + (oh * sh + i) * W + ow * sw + j] += g;
      }
}

/* Fully connected layer as a dense product ("Vectorizing Fully Connected Layers"):
 * y[b,o] = sigma(bias[o] + sum_i x[b,i] w[o,i]). */
void oracle_fc_fwd(const double *x, const double *w, const double *bias, double *y, int B, int I, int O,
                   int relu) {
#pragma omp parallel for schedule(static)
  for (i64 b = 0; b < B; ++b)
    for (i64 o = 0; o < O; ++o) {
      double acc = bias ? bias[o] : 0.0;
      for (i64 i = 0; i < I; ++i) acc += x[b * I + i] * w[o * I + i];
      if (relu && acc < 0.0) acc = 0.0;
      y[b * O + o] = acc;
    }
}

/* dw[o,i] = sum_b dy[b,o] x[b,i];  db[o] = sum_b dy[b,o];  dx[b,i] = sum_o dy[b,o] w[o,i]. */
void oracle_fc_bwd(const double *x, const double *w, const double *dy, double *dw, double *db, double *dx,
                   int B, int I, int O) {
#pragma omp parallel for schedule(static)
  for (i64 o = 0; o < O; ++o) {
    for (i64 i = 0; i < I; ++i) {
      double acc = 0.0;
      for (i64 b = 0; b < B; ++b) acc += dy[b * O + o] * x[b * I + i];
      dw[o * I + i] = acc;
    }
    if (db) {
      double acc = 0.0;
      for (i64 b = 0; b < B; ++b) acc += dy[b * O + o];
      db[o] = acc;
    }
  }
  if (dx) {
#pragma omp parallel for schedule(static)
    for (i64 b = 0; b < B; ++b)
      for (i64 i = 0; i < I; ++i) {
        double acc = 0.0;
        for (i64 o = 0; o < O; ++o) acc += dy[b * O + o] * w[o * I + i];
        dx[b * I + i] = acc;
      }
  }
}

/* Softmax followed by the cross-entropy error (the cost the paper's networks train with), mean over
 * the batch: loss = (1/B) sum_b (logsumexp(z_b) - z_b[label_b]);  dz[b,j] = (softmax(z_b)[j] - [j==label_b])/B. */
double oracle_softmax_loss(const double *z, const int32_t *labels, double *dz, int B, int Cn) {
  double total = 0.0;
  for (i64 b = 0; b < B; ++b) {
    const double *zb = z + b * Cn;
    double m = zb[0];
    for (i64 j = 1; j < Cn; ++j)
      if (zb[j] > m) m = zb[j];
    double se = 0.0;
    for (i64 j = 0; j < Cn; ++j) se += exp(zb[j] - m);
    const double lse = m + log(se);
    total += lse - zb[labels[b]];
    if (dz)
      for (i64 j = 0; j < Cn; ++j) dz[b * Cn + j] = (exp(zb[j] - lse) - (j == labels[b] ? 1.0 : 0.0)) / B;
  }
  return total / B;
}

/* Squared-error cost for the image-to-image networks: loss = 1/(2B) sum (y-t)^2;  dy = (y-t)/B. */
double oracle_l2_loss(const double *y, const double *t, double *dy, i64 count, int B) {
  double total = 0.0;
  for (i64 i = 0; i < count; ++i) {
    const double d = y[i] - t[i];
    total += d * d;
    if (dy) dy[i] = d / B;
  }
  return total / (2.0 * B);
}

/* Plain stochastic gradient descent: w <- w - lr * dw. */
void oracle_sgd_update(double *w, const double *dw, double lr, i64 count) {
  for (i64 i = 0; i < count; ++i) w[i] -= lr * dw[i];
}
