// Internal declarations shared by the vcnn translation units (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/vcnn.h"

namespace vcnn {

// Records a formatted message for vcnn_last_error() and returns `st`.
vcnn_status fail(vcnn_status st, const char* fmt, ...);
// Converts the HIP error state after a launch into a status.
vcnn_status check_launch(const char* what);

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Shape of one convolution layer in the paper's matrix terms: the kernel matrix is M x K, the patch
// matrix K x N, the feature-map matrix M x N (Fig. 2 / Fig. 5: one feature map per row, samples side
// by side).
struct ConvGeom {
  int n, c, h, w, k, r, s, ph, pw, oh, ow;
  int64_t P;      // oh*ow: columns per sample
  int64_t M, K, N;
};

// ---- unroll.hip ---------------------------------------------------------------------------------
// dtype = element type of x and of the patch matrix (im2col); of dx (col2im, whose patch matrix is float)
vcnn_status launch_im2col(const ConvGeom& g, int dtype, const void* x, void* col, hipStream_t st);
vcnn_status launch_col2im(const ConvGeom& g, int dtype, const float* col, void* dx, hipStream_t st);

// ---- conv_small.hip -----------------------------------------------------------------------------
// Correlation of x [n][c][h][w] with the kernel matrix wgt [m][c*r*s] for small layers: one 32 x 32 tile per block,
// the contraction split over its waves, the input rows staged in LDS once.
bool conv_small_applies(int n, int c, int h, int w, int m, int r, int s, int ph, int pw);
vcnn_status launch_conv_small(int dtype, int n, int c, int h, int w, int m, int r, int s, int ph, int pw, const void* x,
                              const void* wgt, const float* bias, void* y, int relu, hipStream_t st);
// Input gradient dx [n][c][h][w] of a small layer from dy [n][m][oh][ow] and the kernels wgt [m][c][r][s]: the
// transposed product and phi_c^{-1} on chip, one sample and four channels per block (fp32 only).
bool conv_small_bwd_applies(int dtype, int n, int c, int h, int w, int m, int r, int s, int ph, int pw);
vcnn_status launch_conv_small_bwd(int n, int c, int h, int w, int m, int r, int s, int ph, int pw,
                                  const void* dy, const void* wgt, void* dx, hipStream_t st);

// ---- gemm.hip -----------------------------------------------------------------------------------
// Generic strided product C(i,j) = act(bias[i] + sum_k A(i,k) B(k,j)), fp32 MFMA.
//   A(i,k) = A[i*a_si + k*a_sk]
//   B(k,j) = B[k*b_sk + jmap_b(j)],  jmap(j) = P ? (j / P)*s_img + (j % P)*s_j : j*s_j
//   C(i,j) = C[i*c_si + jmap_c(j)]
// Exactly one of (a_si, a_sk) and one of (b_sk, b_sj) should be 1 for coalesced loads.
struct GemmArgs {
  const void* A;      // elements of in_dtype
  const void* B;      // elements of in_dtype
  void* C;            // elements of out_dtype
  const float* bias;  // per row i, nullable
  int in_dtype, out_dtype;  // VCNN_F32 | VCNN_BF16 (VCNN_F32 == 0 is the zero-initialised default)
  int M, N, K;
  int64_t a_si, a_sk;
  int64_t b_sk, b_sj, b_simg;
  int b_P;
  int64_t c_si, c_sj, c_simg;
  int c_P;
  int relu;
  // optional: C(i,j) is multiplied by sigma'(.) of activation dact, evaluated from dact_ref (elements of
  // out_dtype, indexed like C: the forward output of that activation)
  int dact;
  const void* dact_ref;
  // optional, small products only: the row sums of A, sum_k A(i,k), written to row_sums[i]
  float* row_sums;
};
vcnn_status launch_gemm_f32(const GemmArgs& a, hipStream_t st);
// true if launch_gemm_f32 takes the small-product kernel (one 32 x 32 tile per block, contraction split over waves)
bool gemm_is_small(const GemmArgs& a);
// The weight-gradient (gw) and input-gradient (gx) products of a fully connected layer in one launch; both small.
vcnn_status launch_fc_bwd_small(const GemmArgs& gw, const GemmArgs& gx, hipStream_t st);

// Filter-gradient product: dW[m][k] = sum_j dY(m,j) * col[k][j] with dY in [N][M][P] layout, contraction
// split over `splits` column ranges whose partial sums are combined in a fixed order.
int bwd_filter_splits(const ConvGeom& g);
size_t bwd_filter_partial_bytes(const ConvGeom& g);
// xin != nullptr (unpadded 1 x 1 layers only): the patch matrix is the input itself, read in place; col is unused
vcnn_status launch_bwd_filter_gemm_f32(const ConvGeom& g, int dtype, const void* dy, const void* col, const void* xin,
                                       float* dw, float* partial, hipStream_t st);

// ---- direct.hip ---------------------------------------------------------------------------------
// Generic correlation out[n][o][y][x] = sum_{i,r,s} wgt(o,i,r,s) * in[n][i][y+r-py][x+s-px] used by the
// direct kernels; wgt(o,i,r,s) = w[o*w_so + i*w_si + tap], tap = r*S+s or, flipped, (R-1-r)*S+(S-1-s).
struct DirectGeom {
  int n, ci, ih, iw, co, oh, ow, r, s, py, px;
  int64_t w_so, w_si;
  int flip;
  int bh, bands, twp, groups;  // band height, number of bands, LDS row pitch, 4-pixel groups per row
};
bool direct_fwd_geom(const ConvGeom& c, DirectGeom* g);
bool direct_bwd_data_geom(const ConvGeom& c, DirectGeom* g);
bool direct_few_out_plan(DirectGeom* g, int* isplit, size_t* partial_bytes);
bool direct_few_in_plan(DirectGeom* g, int* ogroup);
bool direct_filter_grad_plan(const ConvGeom& c, DirectGeom* g, int* slices, size_t* partial_bytes);
vcnn_status launch_direct_few_out(const DirectGeom& g, int dtype, int isplit, const void* in, const void* w,
                                  const float* bias, void* out, float* partial, int relu, hipStream_t st);
vcnn_status launch_direct_few_in(const DirectGeom& g, int dtype, int ogroup, const void* in, const void* w,
                                 const float* bias, void* out, int relu, hipStream_t st, int dact = 0,
                                 const void* dact_ref = nullptr);  // dact / dact_ref: the result is multiplied by sigma'(.) of
                                 // the activation dact (VCNN_ACT_*), evaluated from dact_ref, a tensor of out's shape and type
vcnn_status launch_direct_filter_grad(const DirectGeom& g, int dtype, int slices, const void* x, const void* dy,
                                      float* dw, float* partial, hipStream_t st);

// ---- conv_implicit.hip ----------------------------------------------------------------------------
// Implicit-unroll convolution y = act(bias + W (*) x) on the matrix cores; see the file header.
struct HaloPlan {
  int bm, bn;        // block tile: output maps x consecutive output pixels
  int bk;            // slab depth of the kernel-matrix operand
  int cc;            // input channels staged per chunk
  int nr, wp;        // halo tile rows and row pitch per channel
  int kch;           // taps per chunk, padded to the slab depth
  int tw;            // 0: tiles are runs of bn consecutive pixels; else strips of bn / tw rows x tw columns
  int64_t tiles_per_img;
  size_t lds_bytes;
  bool vec;          // kernel-matrix rows can be fetched 16 bytes at a time
};
bool conv_halo_plan(int n, int c, int h, int w, int m, int r, int s, int ph, int pw, HaloPlan* p);
vcnn_status launch_conv_halo(const HaloPlan& p, int dtype, int n, int c, int h, int w, int m, int r, int s, int ph,
                             int pw, const void* x, const void* wgt, const float* bias, void* y, int relu,
                             hipStream_t st);
struct HaloFilterPlan {
  int bm, bnk;       // block tile: output maps x kernel-matrix columns
  int bp;            // output pixels per staged run
  int ccs, nr, wp;   // channels, rows and row pitch of the halo tile
  int runs_per_img, runs_per_split, splits;
  size_t lds_bytes, partial_bytes;
  bool vec;
  bool vec4_any;     // float dY can be fetched 16 bytes at a time from any dword boundary (every run has >= 4 pixels)
  bool bias_column;  // the last column tile has a spare column: it carries the bias gradient (B operand = 1)
};
bool conv_halo_filter_plan(const ConvGeom& g, HaloFilterPlan* p);
// dbias may be null; with p.bias_column it is produced by the same launches, otherwise the caller computes it
vcnn_status launch_conv_halo_filter(const HaloFilterPlan& p, int dtype, const ConvGeom& g, const void* x, const void* dy,
                                    float* dw, float* dbias, float* partial, hipStream_t st);
struct FewColsPlan {
  int tm, tn;        // 32-row / 32-column tiles of the whole M x K result
  int nr, wp;
  int tw;            // 0: runs of consecutive pixels; else strips of 128 / tw rows x tw columns
  int runs_per_img, total_runs, runs_per_block, blocks;
  bool bias_column;  // the kernel can produce the bias gradient in a spare column of its last tile
  size_t lds_bytes, partial_bytes;
};
bool filter_grad_few_cols_plan(const ConvGeom& g, FewColsPlan* p);
// dbias nullable; when the plan has a bias column and dbias is given, dbias is produced here as well
vcnn_status launch_filter_grad_few_cols(const FewColsPlan& p, int dtype, const ConvGeom& g, const void* x, const void* dy,
                                        float* dw, float* dbias, float* partial, hipStream_t st);
vcnn_status launch_flip_transpose(int dtype, const void* w, void* w2, int M, int C, int RS, hipStream_t st);

// ---- bf16_conv.hip (implicit bf16 kernels) / bf16_mfma.hip (explicit-route bf16 product) ------------
struct HaloBf16Plan {
  int waves_m;       // waves of a block along the output maps
  int waves_n;       // waves of a block along the pixels (same maps: they read the same kernel-matrix fragments);
                     // the remaining 4 / (waves_m * waves_n) split the contraction
  int m16;           // 1: 33..48 maps on 16 x 16 tiles (tm = 3 row tiles, tn in 16-pixel tiles), else 32 x 32 tiles
  int tm;            // row tiles per wave (32-row tiles: 1 for at most 32 maps, else 2)
  int tn;            // column tiles per wave (of 32 pixels, or of 16 with m16)
  int cg, cgc;       // channel groups of 8: total, staged per chunk
  int nchunks;
  int nr, wp;        // halo rows and row pitch (positions of 8 channels) per group
  int uch;           // (group, tap) pairs per chunk, padded to a multiple of 8
  int hpos;          // positions per halo buffer (per term)
  int nbuf;          // halo buffers in LDS (2, or 1 when three planes only fit once)
  int terms;         // 1: bfloat16 operands; 3: float operands as three bfloat16 terms each, six products per step
  size_t lds_bytes;
  size_t x8_bytes, wf_bytes;  // workspace: channel-interleaved input, fragment-ordered kernel matrix
};
struct BwdFilterBf16Plan {
  int bm, splits;
  int64_t chunk;
  size_t dyt_bytes, col_bytes, partial_bytes;
};
// Unpadded 1 x 1 layers of the bf16 variant as plain bf16 products on the NCHW tensors (bf16_pointwise.hip).
struct PointwiseBf16Plan {
  int bm, tiles_m, tiles_p;
};
struct PointwiseFilterBf16Plan {
  int bm, slabs_per_img, units_per_split, splits;
  size_t partial_bytes;
};
// Y[n][rows][P] = act(bias + A[rows][depth] * X[n][depth][P]); A contraction-contiguous and 16-byte aligned
bool pointwise_bf16_plan(int64_t n, int64_t rows, int64_t depth, int64_t P, PointwiseBf16Plan* p);
vcnn_status launch_pointwise_bf16(const PointwiseBf16Plan& p, int n, int rows, int depth, int P, const void* A, const void* X,
                                  const float* bias, void* Y, int relu, hipStream_t st);
bool pointwise_filter_bf16_plan(const ConvGeom& g, PointwiseFilterBf16Plan* p);
vcnn_status launch_pointwise_filter_bf16(const PointwiseFilterBf16Plan& p, const ConvGeom& g, const void* x, const void* dy,
                                         float* dw, float* partial, hipStream_t st);
bool conv_halo_bf16_plan(int n, int c, int h, int w, int m, int r, int s, int ph, int pw, HaloBf16Plan* p, int terms = 1);
// y = act(bias + W (*) x) with W(o, i, q) = wgt[o*w_so + i*w_si + (flip ? r*s-1-q : q)]; the workspace holds
// x8_bytes + wf_bytes
vcnn_status launch_conv_halo_bf16(const HaloBf16Plan& p, int n, int c, int h, int w, int m, int r, int s, int ph, int pw,
                                  const void* x, const void* wgt, int64_t w_so, int64_t w_si, int flip, const float* bias,
                                  void* y, int relu, void* workspace, hipStream_t st, float* y32 = nullptr,
                                  int accumulate = 0);  // y32: float result (added to its contents when accumulate) instead of y
// The same with the two re-laid operands in buffers of the caller (x8_bytes, wf_bytes); a null x or wgt means that its
// buffer already holds that operand from an earlier call.
vcnn_status launch_conv_halo_bf16_prepared(const HaloBf16Plan& p, int n, int c, int h, int w, int m, int r, int s, int ph,
                                           int pw, const void* x, const void* wgt, int64_t w_so, int64_t w_si, int flip,
                                           const float* bias, void* y, int relu, void* x8_buf, void* wf_buf, hipStream_t st,
                                           float* y32, int accumulate);
vcnn_status launch_conv_halo_bf16_terms(const HaloBf16Plan& p, int n, int c, int h, int w, int m, int r, int s, int ph,
                                        int pw, const void* x_terms, size_t x_term_bytes, const void* w_terms,
                                        size_t w_term_bytes, int64_t w_so, int64_t w_si, const float* bias, float* y32,
                                        int relu, void* x8_bufs, void* wf_bufs, hipStream_t st);
struct FilterGradBf16Plan {
  int waves_m, tm, tn;
  int waves_n;       // waves of a block along the kernel-matrix columns (same maps)
  int terms;         // 1: bfloat16 operands; 3: float operands as three bfloat16 terms each, six products per step
  int nbuf;          // halo buffers in LDS (2, or 1 when three planes only fit once)
  int ccs, nr, wp;   // channels, rows and row pitch of the halo tile
  int bh, bp, runs;  // output rows / pixels per run, runs per image
  int ngroups;       // image groups of 8
  int uch, hpos;
  int chunks, chunks_per_split, splits;
  int mt_total;
  size_t lds_bytes, x8n_bytes, dyf_bytes, partial_bytes;
};
bool filter_grad_bf16_plan(const ConvGeom& g, FilterGradBf16Plan* p, int terms = 1);
// workspace: x8n_bytes + dyf_bytes + partial_bytes
// accumulate: dw += the product; the workspace then needs max(partial_bytes, one slice of M*K floats) behind dyf
vcnn_status launch_filter_grad_bf16(const FilterGradBf16Plan& p, const ConvGeom& g, const void* x, const void* dy,
                                    float* dw, void* workspace, hipStream_t st, int accumulate = 0);
// The same with the re-laid operands in buffers of the caller (x8n_bytes, dyf_bytes; null x or dy: already there) and
// the slices in `partial`.
vcnn_status launch_filter_grad_bf16_prepared(const FilterGradBf16Plan& p, const ConvGeom& g, const void* x, const void* dy,
                                             float* dw, void* x8n_buf, void* dyf_buf, float* partial, hipStream_t st,
                                             int accumulate);
vcnn_status launch_filter_grad_bf16_terms(const FilterGradBf16Plan& p, const ConvGeom& g, const void* x_terms,
                                          size_t x_term_bytes, const void* dy_terms, size_t dy_term_bytes, float* dw,
                                          void* x8n_bufs, void* dyf_bufs, float* partial, hipStream_t st);

// ---- split_bf16.hip: fp32 products of large layers as sums of bf16 products (on request only) ------------------------
struct SplitPlan {
  HaloBf16Plan fwd;
  FilterGradBf16Plan filter;
  size_t part_x_bytes, part_w_bytes, part_dy_bytes;  // one bf16 term of x, of w, of dy
  size_t inner_bytes;                                // workspace of the bf16 kernel
  size_t workspace_bytes;
};
bool conv_split_plan(const ConvGeom& g, int pass, SplitPlan* p);
vcnn_status launch_conv_split_fwd(const SplitPlan& p, const ConvGeom& g, const float* x, const float* w, const float* bias,
                                  float* y, int relu, void* workspace, hipStream_t st);
vcnn_status launch_conv_split_filter(const SplitPlan& p, const ConvGeom& g, const float* x, const float* dy, float* dw,
                                     void* workspace, hipStream_t st);
bool bwd_filter_bf16_plan(const ConvGeom& g, BwdFilterBf16Plan* p);
vcnn_status launch_bwd_filter_bf16(const BwdFilterBf16Plan& p, const ConvGeom& g, const void* x, const void* dy, float* dw,
                                   void* workspace, hipStream_t st);

// ---- conv_fold.hip ------------------------------------------------------------------------------------
// Input gradient as the transposed product with phi_c^{-1} applied to each tile on chip (layers with many output
// maps and large kernels, whose patch-matrix gradient would be gigabytes).  workspace: partial_bytes.
struct FoldPlan {
  int tiles_i, tiles_j, rsz, wreg;
  size_t lds_bytes, partial_bytes;
};
bool bwd_data_fold_plan(const ConvGeom& g, FoldPlan* p);
vcnn_status launch_bwd_data_fold(const FoldPlan& p, int dtype, const ConvGeom& g, const void* w, const void* dy, void* dx,
                                 float* partial, hipStream_t st, int dact = 0, const void* dact_ref = nullptr);

// ---- conv_taps.hip --------------------------------------------------------------------------------------
// One-map layers over many channels with the kernel's taps as the rows of the product (see the file header).
bool conv_taps_applies(const ConvGeom& g);
size_t conv_taps_fwd_bytes(const ConvGeom& g);             // workspace of the forward pass (Z)
size_t conv_taps_filter_bytes(const ConvGeom& g, int dtype);  // workspace of the kernel gradient
vcnn_status launch_conv_taps_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, const float* bias, void* y,
                                 int relu, float* z, hipStream_t st);
vcnn_status launch_conv_taps_filter(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* workspace,
                                    hipStream_t st);

// ---- fft_conv.hip -------------------------------------------------------------------------------------
// Forward pass of layers with r x 1 or 1 x s kernels through the Fourier domain (comparison route).
// workspace: xf_bytes + wf_bytes + yf_bytes.
struct FftPlan {
  int along_w, len, taps, pad, out_len, other, Q, L, logL, LP, sb;
  size_t xf_bytes, wf_bytes, yf_bytes;
};
bool conv_fft_plan(const ConvGeom& g, FftPlan* p);
vcnn_status launch_conv_fft(const FftPlan& p, int dtype, const ConvGeom& g, const void* x, const void* w, const float* bias,
                            void* y, int relu, void* workspace, hipStream_t st);

// out[i] = act(bias[(i / plane) % maps] + sum_s partial[s][i]), slices added in ascending order (bias nullable)
vcnn_status launch_sum_slices(const float* partial, const float* bias, void* out, int out_dtype, int64_t count,
                              int splits, int64_t plane, int maps, int relu, hipStream_t st);
// partial is [splits][rows][cols + 1]: main[r][c] = sum_s partial[s][r][c] for c < cols, last[r] = sum_s partial[s][r][cols]
vcnn_status launch_sum_slices_split(const float* partial, float* main, float* last, int64_t rows, int cols, int splits,
                                    hipStream_t st);

// ---- pointwise.hip ------------------------------------------------------------------------------
// dtype selects the element type (VCNN_F32 / VCNN_BF16) of the activation tensors passed as void*.
size_t bias_grad_partial_bytes(const ConvGeom& g);
vcnn_status launch_bias_grad(const ConvGeom& g, int dtype, const void* dy, float* db, float* partial, hipStream_t st);
vcnn_status launch_relu_fwd(int dtype, size_t count, const void* x, void* y, hipStream_t st);
vcnn_status launch_relu_bwd(int dtype, size_t count, const void* ref, const void* dy, void* dx, hipStream_t st);
// tanh / sigmoid: dy == nullptr -> forward from a = x; else backward from a = forward output
vcnn_status launch_smooth_act(int act, int dtype, size_t count, const void* a, const void* dy, void* out, hipStream_t st);
// bias (per map, nullable) and act (VCNN_ACT_*): the epilogue of the pooling layer, forward only
vcnn_status launch_avgpool(const vcnn_pool_desc& d, int oh, int ow, const void* src, void* dst, bool backward,
                           const float* bias, int act, hipStream_t st);
vcnn_status launch_pool_fwd(const vcnn_pool_desc& d, int oh, int ow, const void* x, void* y, int32_t* argmax,
                            const float* bias, int act, hipStream_t st);
// act / ref: optional activation derivative folded into the store (ref = the pooling input, indexed like dx)
vcnn_status launch_pool_bwd(const vcnn_pool_desc& d, int oh, int ow, const void* dy, const int32_t* argmax, void* dx,
                            int act, const void* ref,
                            hipStream_t st);
vcnn_status launch_col_sum(int dtype, int rows, int cols, const void* a, float* out, hipStream_t st);  // out[c] = sum_r a[r][c]
vcnn_status launch_softmax_loss_f32(int batch, int classes, const float* z, const int32_t* labels, float* loss,
                                    float* dz, hipStream_t st);
vcnn_status launch_l2_loss(int dtype, size_t count, int batch, const void* y, const float* t, float* loss, void* dy,
                           hipStream_t st);
vcnn_status launch_sgd_f32(size_t count, float lr, float* w, const float* dw, hipStream_t st);
// up to kSgdBatch tensors per launch; first[t] = index of tensor t's first block, first[tensors] = grid size
static constexpr int kSgdBatch = 16;
struct SgdBatch {
  float* w[kSgdBatch];
  const float* dw[kSgdBatch];
  void* w16[kSgdBatch];  // optional bfloat16 copy of the updated tensor
  size_t count[kSgdBatch];
  unsigned first[kSgdBatch + 1];
  int tensors;
  float lr;
};
vcnn_status launch_sgd_multi(const SgdBatch& a, hipStream_t st);
vcnn_status launch_f32_to_bf16(size_t count, const float* src, uint16_t* dst, hipStream_t st);
vcnn_status launch_bf16_to_f32(size_t count, const uint16_t* src, float* dst, hipStream_t st);

}  // namespace vcnn
