/*
 * vcnn - the vectorized CNN layer path of Ren & Xu, "On Vectorization of Deep Convolutional Neural
 * Networks for Vision Tasks" (AAAI 2015), as hand-written HIP kernels for AMD CDNA4 (gfx950).
 *
 * The convolution layer is computed the way the paper formulates it: the input is unrolled into a
 * dense patch matrix (the operator phi_c), all kernels are stacked as rows of a second matrix, and
 * one matrix product yields every feature map of every sample of the mini-batch (Eq. 2 and Eq. 4).
 * Back-propagation multiplies by the transposed matrices and folds the patch-matrix gradient back
 * with the many-to-one operator phi_c^{-1}.
 *
 * Conventions common to every call
 *   - Plain C ABI.  Every call returns a vcnn_status; VCNN_OK is 0, errors are negative.  Argument
 *     validation happens before anything is enqueued and needs no GPU.  vcnn_last_error() returns a
 *     thread-local text describing the last failure on the calling thread.
 *   - Every data pointer is a DEVICE pointer owned by the caller.  Descriptor pointers and the
 *     out-parameters of the *_shape / *_bytes queries are HOST pointers.  The library never
 *     allocates, frees or retains device memory and never synchronises: it only enqueues kernels on
 *     `stream` (a hipStream_t passed as void*; NULL means the default stream).
 *   - Tensors are dense and contiguous.  Activations are [N][C][H][W]; convolution kernels are
 *     [K][C][R][S] (K output maps); fully connected weights are [O][I].
 *   - dtype VCNN_F32: every tensor is float.  dtype VCNN_BF16: x, w, y, dy, dx are bfloat16
 *     (16-bit, round-to-nearest-even on store); bias, dw, dbias, losses and all accumulation are float.
 *   - "Convolution" is cross-correlation (no kernel flip), which is what multiplying the kernel
 *     rows by the patch columns computes.  Padding is zero extension.  Only stride 1 is built
 *     (the paper's networks use stride 1 throughout); other strides return VCNN_ERR_UNSUPPORTED.
 *   - Results are bit-identical from run to run: no floating-point atomics are used anywhere.
 *   - Workspaces must be 256-byte aligned.
 */
#ifndef VCNN_H
#define VCNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t vcnn_status;
enum {
  VCNN_OK = 0,
  VCNN_ERR_NULL = -1,        /* a required pointer is NULL */
  VCNN_ERR_SHAPE = -2,       /* non-positive dimension, kernel larger than padded input, window larger than input */
  VCNN_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or too small */
  VCNN_ERR_UNSUPPORTED = -4, /* dtype / stride / activation combination that is not built */
  VCNN_ERR_HIP = -5          /* the HIP runtime refused a launch; see vcnn_last_error() */
};

enum { VCNN_F32 = 0, VCNN_BF16 = 1 };
enum { VCNN_ACT_NONE = 0, VCNN_ACT_RELU = 1, VCNN_ACT_TANH = 2, VCNN_ACT_SIGMOID = 3 };  /* sigma of Eq. 1 */
enum { VCNN_POOL_MAX = 0, VCNN_POOL_AVG = 1 };  /* the operation of phi_p ("Vectorizing Pooling") */
enum { VCNN_PASS_FWD = 0, VCNN_PASS_BWD_FILTER = 1, VCNN_PASS_BWD_DATA = 2 };

/* How the convolution calls realise the unroll.  EXPLICIT materialises the patch matrix in the
 * workspace (phi_c as a kernel of its own, then a matrix product); IMPLICIT forms the patch-matrix
 * tiles on the fly inside the product.  AUTO picks per shape.  FOLD is AUTO except that the input gradient
 * takes, wherever the layer allows it, the transposed product with phi_c^{-1} applied to every tile of the
 * patch-matrix gradient on chip (AUTO uses that route only where it is the fastest).  FFT is AUTO except that the
 * forward pass of layers with one-dimensional kernels (r x 1 or 1 x s, at least 8 taps, no padding across the
 * kernel) goes through the Fourier domain - the alternative the paper's related-work paragraph names ("FFT
 * speedup"), kept as a comparison: AUTO never takes it.  SPLIT is AUTO except that the forward pass and the kernel
 * gradient of fp32 layers with more than 4 maps and channels compute their products (Eq. 1 / Eq. 2) as sums of
 * bfloat16 products: every float operand is, exactly, a sum of three bfloat16 terms, and the six largest of the nine
 * term products, accumulated in float, carry the product to within float rounding.  The result stays within the
 * float tolerance; the matrix cores multiply bfloat16 sixteen times as fast as float.  AUTO never takes it. */
enum { VCNN_ALGO_AUTO = 0, VCNN_ALGO_EXPLICIT = 1, VCNN_ALGO_IMPLICIT = 2, VCNN_ALGO_FOLD = 3, VCNN_ALGO_FFT = 4,
       VCNN_ALGO_SPLIT = 5 };

typedef struct {
  int32_t n, c, h, w;                         /* input: batch, channels, height, width */
  int32_t k, r, s;                            /* output maps, kernel height, kernel width */
  int32_t pad_h, pad_w, stride_h, stride_w;   /* zero padding per side; stride (must be 1) */
  int32_t dtype;                              /* VCNN_F32 | VCNN_BF16 */
  int32_t act;                                /* VCNN_ACT_* applied by the forward pass (ReLU inside the product's
                                                 epilogue, tanh / sigmoid by an element-wise pass over y) */
} vcnn_conv_desc;

typedef struct {
  int32_t n, c, h, w;                         /* input */
  int32_t win_h, win_w, stride_h, stride_w;   /* window and stride; no padding */
  int32_t dtype;
  int32_t mode;                               /* VCNN_POOL_MAX (0) | VCNN_POOL_AVG */
} vcnn_pool_desc;

const char* vcnn_status_string(vcnn_status st);
const char* vcnn_last_error(void);
/* Library version as major*10000 + minor*100 + patch. */
int32_t vcnn_version(void);
/* Process-wide choice of VCNN_ALGO_* for the convolution calls (default AUTO).  Returns VCNN_ERR_UNSUPPORTED
 * for an unknown value.  Meant for A/B measurements; every choice computes the same function. */
vcnn_status vcnn_set_conv_algo(int32_t algo);

/* Output size of the layer of Eq. 1: oh = (h + 2*pad_h - r)/stride_h + 1, likewise ow. */
vcnn_status vcnn_conv_out_shape(const vcnn_conv_desc* d, int32_t* oh, int32_t* ow);
/* Bytes of workspace the given pass needs for this descriptor (may be 0). */
vcnn_status vcnn_conv_workspace_bytes(const vcnn_conv_desc* d, int32_t pass, size_t* bytes);

/* phi_c (Eq. 2; mini-batch form Eq. 4): col[(c*R+r)*S+s][(n*OH+oh)*OW+ow] = xpad[n][c][oh+r-pad_h][ow+s-pad_w].
 * col is a dense [C*R*S][N*OH*OW] matrix of the descriptor's dtype.  Pure data movement. */
vcnn_status vcnn_im2col(const vcnn_conv_desc* d, const void* x, void* col, void* stream);
/* phi_c^{-1} (back-propagation paragraph of "Vectorizing Convolution"): dx[n][c][h][w] = sum over the
 * entries of col that phi_c copied from that pixel, added in ascending (r, s) order.  col is float. */
vcnn_status vcnn_col2im(const vcnn_conv_desc* d, const float* col, void* dx, void* stream);

/* Forward layer, Eq. 1/2/4: y[n][k][oh][ow] = act(bias[k] + sum_{c,r,s} w[k][c][r][s]*xpad[n][c][oh+r-pad_h][ow+s-pad_w]).
 * bias may be NULL (treated as zero). */
vcnn_status vcnn_conv_fwd(const vcnn_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                          void* workspace, size_t workspace_bytes, void* stream);
/* Kernel and bias gradients: dw = dy_matrix * phi_c(x)^T, dbias[k] = sum dy[:,k,:,:] (dbias may be NULL).
 * dy is the gradient w.r.t. the layer's pre-activation: when act was fused in forward the caller
 * applies vcnn_act_bwd to dy first. */
vcnn_status vcnn_conv_bwd_filter(const vcnn_conv_desc* d, const void* x, const void* dy, float* dw, float* dbias,
                                 void* workspace, size_t workspace_bytes, void* stream);
/* vcnn_conv_bwd_filter for callers that cannot allocate device memory or size a workspace: code under HIP graph
 * capture, tight serving or fine-tuning loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels, bit for bit; the partial sums live in a fixed array inside the library's code object
 * (vcnn_conv_bwd_filter_noalloc_limit() bytes, 32 MiB, held by every GPU the library runs on until the process
 * ends) instead of a caller workspace.  The call allocates and frees nothing.  A layer whose pass needs more
 * (vcnn_conv_workspace_bytes(d, VCNN_PASS_BWD_FILTER) > limit) is rejected with VCNN_ERR_WORKSPACE before anything
 * is enqueued.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or host threads) race; calls ordered on one stream do not.  The first call on each device looks the
 * array's address up and should be made outside a stream capture. */
size_t vcnn_conv_bwd_filter_noalloc_limit(void);
vcnn_status vcnn_conv_bwd_filter_noalloc(const vcnn_conv_desc* d, const void* x, const void* dy, float* dw,
                                         float* dbias, void* stream);
/* Input gradient: dx = phi_c^{-1}(W^T * dy_matrix).  Same convention for dy as above. */
vcnn_status vcnn_conv_bwd_data(const vcnn_conv_desc* d, const void* w, const void* dy, void* dx, void* workspace,
                               size_t workspace_bytes, void* stream);
/* vcnn_conv_bwd_data with the next step of the delta recursion ("Vectorizing Convolution", back-propagation paragraph;
 * Eq. 1's sigma) folded into its store, as in vcnn_pool_bwd_act: x, this layer's input, is the forward OUTPUT of the
 * activation act_below applied by the layer below, and dx = phi_c^{-1}(W^T * dy_matrix) * sigma'(.) evaluated from x
 * (ReLU: x > 0; tanh: 1 - x^2; sigmoid: x (1 - x)), i.e. the gradient w.r.t. that layer's pre-activation; the separate
 * vcnn_act_bwd call is then not needed.  x has the shape and dtype of dx ([n][c][h][w], device).  act_below ==
 * VCNN_ACT_NONE is vcnn_conv_bwd_data (x is not read and may be NULL).  Same workspace as vcnn_conv_bwd_data
 * (VCNN_PASS_BWD_DATA); VCNN_ERR_UNSUPPORTED for an unknown activation, VCNN_ERR_NULL for a missing tensor. */
vcnn_status vcnn_conv_bwd_data_act(const vcnn_conv_desc* d, int32_t act_below, const void* x, const void* w, const void* dy,
                                   void* dx, void* workspace, size_t workspace_bytes, void* stream);

/* Max pooling ("Vectorizing Pooling", phi_p with the max operation).  Output size
 * floor((h-win_h)/stride_h)+1 by floor((w-win_w)/stride_w)+1.  argmax[n][c][oh][ow] is the int32 flat
 * index h*W+w, inside the (n,c) input plane, of the window's maximum; among equal maxima the lowest
 * index is recorded.  Inputs are assumed finite. */
vcnn_status vcnn_pool_out_shape(const vcnn_pool_desc* d, int32_t* oh, int32_t* ow);
vcnn_status vcnn_pool_fwd(const vcnn_pool_desc* d, const void* x, void* y, int32_t* argmax, void* stream);
/* Routes each output gradient to the recorded position; overlapping windows that recorded the same
 * position are summed in ascending window order.  Every element of dx is written.
 * Average pooling (mode VCNN_POOL_AVG): y = mean of the window, argmax is not used and may be NULL in both
 * calls; the backward pass is the exact transpose, dx[i] = sum over the windows covering i of dy / (win_h*win_w)
 * (for windows that tile the plane: the nearest-neighbour upscaling of dy the paper back-propagates with). */
vcnn_status vcnn_pool_bwd(const vcnn_pool_desc* d, const void* dy, const int32_t* argmax, void* dx, void* stream);
/* The pooling layer of Eq. 3 ("Vectorizing Pooling"): y = sigma(phi_p(x) + b), phi_p the max or the mean of each
 * window (d->mode), b one float per feature map (bias[c], NULL = zero), sigma = act (VCNN_ACT_*).  Shapes, argmax
 * and tie rule as in vcnn_pool_fwd, which is this call with no bias and VCNN_ACT_NONE. */
vcnn_status vcnn_pool_layer_fwd(const vcnn_pool_desc* d, int32_t act, const void* x, const float* bias, void* y,
                                int32_t* argmax, void* stream);
/* Gradients of that layer from its output y and dy = dL/dy: delta = dy * sigma'(.) evaluated from y (as in
 * vcnn_act_bwd), dbias[c] = sum of delta over samples and pixels (NULL: not computed), dx = delta routed back
 * through phi_p as in vcnn_pool_bwd.  workspace: device memory of at least vcnn_pool_layer_workspace_bytes (holds
 * delta and partial sums; contents undefined afterwards; may be NULL when act is VCNN_ACT_NONE and dbias NULL).
 * y is not read when act is VCNN_ACT_NONE.  VCNN_ERR_WORKSPACE if the workspace is too small. */
vcnn_status vcnn_pool_layer_workspace_bytes(const vcnn_pool_desc* d, size_t* bytes);
vcnn_status vcnn_pool_layer_bwd(const vcnn_pool_desc* d, int32_t act, const void* y, const void* dy,
                                const int32_t* argmax, float* dbias, void* dx, void* workspace, size_t workspace_bytes,
                                void* stream);
/* vcnn_pool_bwd with the next step of the delta recursion folded into its store: the pooling input x is the
 * forward OUTPUT of the activation act_below (sigma of Eq. 1, applied by the layer below), and
 * dx = pool_bwd(dy) * sigma'(.) evaluated from x (ReLU: x > 0; tanh: 1 - x^2; sigmoid: x (1 - x)), i.e. the
 * gradient w.r.t. that layer's pre-activation; the separate vcnn_act_bwd call is then not needed.  x has the
 * shape and dtype of dx.  act_below == VCNN_ACT_NONE is vcnn_pool_bwd (x is not read). */
vcnn_status vcnn_pool_bwd_act(const vcnn_pool_desc* d, int32_t act_below, const void* x, const void* dy,
                              const int32_t* argmax, void* dx, void* stream);

/* Element-wise sigma of Eq. 1.  ReLU: fwd y = max(x, 0); bwd dx = ref > 0 ? dy : 0, where ref may be
 * either the forward input or the forward output (they are positive at the same places).
 * tanh / sigmoid: fwd y = tanh(x) / 1/(1+exp(-x)); bwd takes ref = the forward OUTPUT y:
 * dx = dy (1 - y^2) / dy y (1 - y).  y == x and dx == dy (in place) are allowed. */
vcnn_status vcnn_act_fwd(int32_t act, int32_t dtype, size_t count, const void* x, void* y, void* stream);
vcnn_status vcnn_act_bwd(int32_t act, int32_t dtype, size_t count, const void* ref, const void* dy, void* dx,
                         void* stream);

/* Fully connected layer as a dense matrix product ("Vectorizing Fully Connected Layers"):
 * y[b][o] = act(bias[o] + sum_i x[b][i]*w[o][i]);  x is [batch][in_f], w [out_f][in_f], y [batch][out_f]. */
vcnn_status vcnn_fc_fwd(int32_t dtype, int32_t batch, int32_t in_f, int32_t out_f, int32_t act, const void* x,
                        const void* w, const float* bias, void* y, void* stream);
/* dw[o][i] = sum_b dy[b][o]*x[b][i];  dbias[o] = sum_b dy[b][o];  dx[b][i] = sum_o dy[b][o]*w[o][i].
 * Each of dw, dbias, dx may be NULL and is then not computed (so the parameter gradients and the input
 * gradient can be issued on different streams); x is read only for dw, w only for dx.  dy is w.r.t. the
 * pre-activation.  Needs no workspace. */
vcnn_status vcnn_fc_bwd(int32_t dtype, int32_t batch, int32_t in_f, int32_t out_f, const void* x, const void* w,
                        const void* dy, float* dw, float* dbias, void* dx, void* stream);
/* vcnn_fc_bwd with the derivative of the activation below folded into the input gradient's store (same
 * convention as vcnn_pool_bwd_act): x, the layer's input, is the forward output of act_below and
 * dx[b][i] = (sum_o dy[b][o]*w[o][i]) * sigma'(.) from x[b][i]; dw and dbias as in vcnn_fc_bwd.  x is then read for
 * dx as well.  When dw and dx are both requested and the products are small (the layers of the experiments at
 * their batch sizes), both - and dbias - come out of one launch.  act_below == VCNN_ACT_NONE is vcnn_fc_bwd. */
vcnn_status vcnn_fc_bwd_act(int32_t dtype, int32_t batch, int32_t in_f, int32_t out_f, int32_t act_below,
                            const void* x, const void* w, const void* dy, float* dw, float* dbias, void* dx,
                            void* stream);

/* Softmax + cross-entropy cost, mean over the batch: loss = (1/B) sum_b (logsumexp(z_b) - z_b[label_b]),
 * dlogits[b][j] = (softmax(z_b)[j] - [j == label_b]) / B.  loss is a device scalar; dlogits may be NULL.
 * Precondition: 0 <= labels[b] < classes.  A label outside that range is never used as an index: the loss and
 * that sample's row of dlogits come out as NaN, and the call still returns VCNN_OK (the labels live on the device). */
vcnn_status vcnn_softmax_loss(int32_t batch, int32_t classes, const float* logits, const int32_t* labels,
                              float* loss, float* dlogits, void* stream);
/* Squared-error cost for the image-to-image networks: loss = 1/(2*batch) * sum (y-t)^2, dy = (y-t)/batch.
 * y and dy follow dtype; target and loss are float.  loss and dy may each be NULL. */
vcnn_status vcnn_l2_loss(int32_t dtype, size_t count, int32_t batch, const void* y, const float* target,
                         float* loss, void* dy, void* stream);
/* Plain SGD on float parameters: w[i] -= lr * dw[i]. */
vcnn_status vcnn_sgd_update(size_t count, float lr, float* w, const float* dw, void* stream);
/* The same update for `tensors` parameter tensors in one launch (the experiments' networks have 4 to 10):
 * w[t][i] -= lr * dw[t][i] for i < counts[t].  counts, w, dw and w_bf16 are HOST arrays of length `tensors`
 * holding element counts and DEVICE pointers; they are read before the call returns.  w_bf16 may be NULL;
 * a non-NULL w_bf16[t] receives the updated tensor rounded to bfloat16 (the working copy of the bf16
 * variant).  Tensors with count 0 are skipped. */
vcnn_status vcnn_sgd_update_multi(int32_t tensors, const size_t* counts, float* const* w, const float* const* dw,
                                  void* const* w_bf16, float lr, void* stream);
/* Rounds a float tensor to bfloat16 (nearest even) and back: dst_bf16[i] = bf16(src[i]);  src_f32[i] = float(bf16). */
vcnn_status vcnn_f32_to_bf16(size_t count, const float* src, void* dst, void* stream);
vcnn_status vcnn_bf16_to_f32(size_t count, const void* src, float* dst, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VCNN_H */
