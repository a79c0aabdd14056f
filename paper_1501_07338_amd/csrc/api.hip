// C-ABI entry points: argument validation, shape algebra, workspace layout and kernel selection.
// Validation never touches the HIP runtime, so error paths can be exercised on a host without a GPU.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "common.h"

namespace vcnn {

static thread_local char g_err[512] = "";
static std::atomic<int> g_conv_algo{VCNN_ALGO_AUTO};

vcnn_status fail(vcnn_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

vcnn_status check_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return VCNN_OK;
  return fail(VCNN_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

static inline size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

static vcnn_status make_geom(const vcnn_conv_desc* d, ConvGeom* g) {
  if (!d) return fail(VCNN_ERR_NULL, "conv descriptor is NULL");
  if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0)
    return fail(VCNN_ERR_SHAPE, "conv: non-positive dimension (n=%d c=%d h=%d w=%d k=%d r=%d s=%d)", d->n, d->c, d->h,
                d->w, d->k, d->r, d->s);
  if (d->pad_h < 0 || d->pad_w < 0) return fail(VCNN_ERR_SHAPE, "conv: negative padding");
  if (d->stride_h <= 0 || d->stride_w <= 0) return fail(VCNN_ERR_SHAPE, "conv: non-positive stride");
  if (d->r > d->h + 2 * d->pad_h || d->s > d->w + 2 * d->pad_w)
    return fail(VCNN_ERR_SHAPE, "conv: kernel %dx%d larger than padded input %dx%d", d->r, d->s, d->h + 2 * d->pad_h,
                d->w + 2 * d->pad_w);
  if (d->dtype != VCNN_F32 && d->dtype != VCNN_BF16) return fail(VCNN_ERR_UNSUPPORTED, "conv: unknown dtype %d", d->dtype);
  if (d->act < VCNN_ACT_NONE || d->act > VCNN_ACT_SIGMOID)
    return fail(VCNN_ERR_UNSUPPORTED, "conv: unknown activation %d", d->act);
  if (d->stride_h != 1 || d->stride_w != 1)
    return fail(VCNN_ERR_UNSUPPORTED, "conv: only stride 1 is built (got %dx%d)", d->stride_h, d->stride_w);
  g->n = d->n, g->c = d->c, g->h = d->h, g->w = d->w, g->k = d->k, g->r = d->r, g->s = d->s;
  g->ph = d->pad_h, g->pw = d->pad_w;
  g->oh = d->h + 2 * d->pad_h - d->r + 1;
  g->ow = d->w + 2 * d->pad_w - d->s + 1;
  g->P = (int64_t)g->oh * g->ow;
  g->M = d->k;
  g->K = (int64_t)d->c * d->r * d->s;
  g->N = (int64_t)d->n * g->P;
  if (g->N > 0x7fffffffLL || g->K > 0x7fffffffLL || (int64_t)d->n * d->c * d->h * d->w > 0x7fffffffLL * 4)
    return fail(VCNN_ERR_UNSUPPORTED, "conv: problem too large (N=%lld K=%lld)", (long long)g->N, (long long)g->K);
  return VCNN_OK;
}

static vcnn_status check_dtype(int32_t dtype, const char* what) {
  if (dtype == VCNN_F32 || dtype == VCNN_BF16) return VCNN_OK;
  return fail(VCNN_ERR_UNSUPPORTED, "%s: unknown dtype %d", what, dtype);
}

static vcnn_status check_ws(const void* ws, size_t have, size_t need, const char* what) {
  if (need == 0) return VCNN_OK;
  if (!ws) return fail(VCNN_ERR_WORKSPACE, "%s: workspace is NULL but %zu bytes are needed", what, need);
  if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(VCNN_ERR_WORKSPACE, "%s: workspace is not 256-byte aligned", what);
  if (have < need) return fail(VCNN_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", what, have, need);
  return VCNN_OK;
}

// The 1x1, unpadded layer's patch matrix is the input itself (per sample), so no unroll is needed.
static bool is_pointwise(const ConvGeom& g) { return g.r == 1 && g.s == 1 && g.ph == 0 && g.pw == 0; }

static size_t col_bytes(const ConvGeom& g) { return align256((size_t)g.K * g.N * sizeof(float)); }

// The input gradient as a correlation over all H x W input pixels multiplies the zero border of a
// 'valid' layer too and puts the input-channel count on the matrix-core row axis, so it can cost more
// matrix-core work than the explicit route (transposed product, then phi_c^{-1}), which instead pays
// for writing and re-reading the patch-matrix gradient.  Estimated times, in seconds, with the rates
// these kernels sustain on MI355X (about 100 TFLOP/s of fp32 MFMA work, 2.5 TB/s through HBM).
static bool halo_bwd_data_pays(const ConvGeom& g, const HaloPlan& hp) {
  const double mfma_rate = 100e12, hbm_rate = 2.5e12;
  const double halo_flops = 2.0 * (double)ceil_div(g.c, hp.bm) * hp.bm * ((double)g.k * g.r * g.s) *
                            ((double)g.n * ceil_div((int64_t)g.h * g.w, hp.bn) * hp.bn);
  const double exp_flops = 2.0 * (double)ceil_div(g.K, 128) * 128 * (double)ceil_div(g.M, 32) * 32 * (double)g.N;
  const double col_traffic = 2.0 * (double)g.K * (double)g.N * sizeof(float);
  return halo_flops / mfma_rate < exp_flops / mfma_rate + 1.3 * col_traffic / hbm_rate;
}

// The same correlation against the fused route (transposed product with phi_c^{-1} per tile on chip), which executes
// exactly the nominal flops but pays a fixed fold per 128 x 128 tile: per tile about 4.1 us per 16 output maps of
// contraction plus 8 us, 1024 tiles resident at once (measured on cfg5 c2 and c3).
static bool fold_beats_halo(const ConvGeom& g, const HaloPlan& hp, const FoldPlan& fp) {
  const double halo_flops = 2.0 * (double)ceil_div(g.c, hp.bm) * hp.bm * ((double)g.k * g.r * g.s) *
                            ((double)g.n * ceil_div((int64_t)g.h * g.w, hp.bn) * hp.bn);
  const double halo_s = halo_flops / 100e12;
  const double tiles = (double)g.n * fp.tiles_i * fp.tiles_j;
  const double fold_s = tiles * (4.1e-6 * (double)ceil_div(g.M, 16) + 8e-6) / 1024.0;
  return fold_s < halo_s;
}

// Which realisation a pass uses for a given shape.  The same decision drives the workspace query and
// the launch, so the two always agree.
enum Path { PATH_EXPLICIT, PATH_POINTWISE, PATH_FEW_OUT, PATH_FEW_IN, PATH_DIRECT_FILTER, PATH_HALO, PATH_HALO_FILTER, PATH_HALO_BF16, PATH_FILTER_BF16, PATH_HALO_FILTER_BF16, PATH_FEW_COLS_FILTER, PATH_SMALL, PATH_SMALL_BWD, PATH_FOLD, PATH_FFT, PATH_TAPS, PATH_POINTWISE_BF16, PATH_SPLIT };
struct Plan {
  Path path;
  DirectGeom dg;
  HaloPlan hp;
  HaloFilterPlan hfp;
  HaloBf16Plan hb;
  BwdFilterBf16Plan fb;
  FilterGradBf16Plan hfb;
  FewColsPlan fcp;
  FoldPlan fold;
  FftPlan fft;
  PointwiseBf16Plan pwb;
  PointwiseFilterBf16Plan pwf;
  SplitPlan sp;
  int split;        // channel slices (few-out), output-map group size (few-in) or batch slices (filter gradient)
  size_t partial_bytes;
  size_t workspace_bytes;
  size_t bias_offset;  // filter-gradient pass: where the bias-gradient partial sums live in the workspace
};

static Plan make_plan(const ConvGeom& g, int pass, int dtype) {
  Plan p{};
  p.path = PATH_EXPLICIT;
  const int algo = g_conv_algo.load();
  const bool allow_direct = algo != VCNN_ALGO_EXPLICIT;
  // FOLD only re-routes the input gradient, FFT only the forward pass of layers with one-dimensional kernels
  const bool automatic = algo == VCNN_ALGO_AUTO || algo == VCNN_ALGO_FOLD || algo == VCNN_ALGO_FFT || algo == VCNN_ALGO_SPLIT;
  if (algo == VCNN_ALGO_SPLIT && dtype == VCNN_F32 && pass != VCNN_PASS_BWD_DATA && conv_split_plan(g, pass, &p.sp)) {
    p.path = PATH_SPLIT;  // float products as sums of bfloat16 products
    p.workspace_bytes = align256(p.sp.workspace_bytes);
    if (pass == VCNN_PASS_BWD_FILTER) {
      p.bias_offset = p.workspace_bytes;
      p.workspace_bytes += align256(bias_grad_partial_bytes(g));
    }
    return p;
  }
  if (algo == VCNN_ALGO_FFT && pass == VCNN_PASS_FWD && conv_fft_plan(g, &p.fft)) {
    p.path = PATH_FFT;
    p.workspace_bytes = p.fft.xf_bytes + p.fft.wf_bytes + p.fft.yf_bytes;
    return p;
  }
  // bf16 variant, default route: the bf16 matrix-core kernels wherever the layer has enough maps / channels
  const bool bf16_mfma = dtype == VCNN_BF16 && automatic;
  // unpadded 1 x 1 layers: three plain bf16 products on the tensors as they are stored
  if (bf16_mfma && is_pointwise(g)) {
    if (pass == VCNN_PASS_FWD && pointwise_bf16_plan(g.n, g.k, g.c, g.P, &p.pwb)) {
      p.path = PATH_POINTWISE_BF16;
      return p;
    }
    if (pass == VCNN_PASS_BWD_DATA && pointwise_bf16_plan(g.n, g.c, g.k, g.P, &p.pwb)) {
      p.path = PATH_POINTWISE_BF16;
      p.workspace_bytes = align256((size_t)g.k * g.c * 2);  // the transposed kernel matrix
      return p;
    }
    if (pass == VCNN_PASS_BWD_FILTER && pointwise_filter_bf16_plan(g, &p.pwf)) {
      p.path = PATH_POINTWISE_BF16;
      p.workspace_bytes = align256(p.pwf.partial_bytes);
      p.bias_offset = p.workspace_bytes;
      p.workspace_bytes += align256(bias_grad_partial_bytes(g));
      return p;
    }
  }
  // (other 1x1 layers included: they are a plain bf16 product through the same kernel)
  // (a single map over many channels is faster as the taps-as-rows product below, in bf16 storage as well)
  if (bf16_mfma && pass == VCNN_PASS_FWD && (g.k > 4 || g.c >= 64) && !conv_taps_applies(g) &&
      conv_halo_bf16_plan(g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, &p.hb)) {
    p.path = PATH_HALO_BF16;
    p.workspace_bytes = p.hb.x8_bytes + p.hb.wf_bytes;
    return p;
  }
  // (at most four maps would fill one channel group of eight: the float matrix-core kernel below reads them unpadded)
  if (bf16_mfma && pass == VCNN_PASS_BWD_DATA && !(algo == VCNN_ALGO_FOLD && bwd_data_fold_plan(g, &p.fold)) && g.c > 4 &&
      g.k > 4 && g.r - 1 - g.ph >= 0 && g.s - 1 - g.pw >= 0 &&
      conv_halo_bf16_plan(g.n, g.k, g.oh, g.ow, g.c, g.r, g.s, g.r - 1 - g.ph, g.s - 1 - g.pw, &p.hb)) {
    p.path = PATH_HALO_BF16;
    p.workspace_bytes = p.hb.x8_bytes + p.hb.wf_bytes;
    return p;
  }
  // (a single map over many channels is faster as the taps-as-rows product below, as in the forward pass)
  if (bf16_mfma && pass == VCNN_PASS_BWD_FILTER && (g.k > 4 || g.c >= 64) && g.c > 4 && !conv_taps_applies(g) &&
      filter_grad_bf16_plan(g, &p.hfb)) {
    p.path = PATH_HALO_FILTER_BF16;
    p.workspace_bytes = p.hfb.x8n_bytes + p.hfb.dyf_bytes + align256(p.hfb.partial_bytes);
    p.bias_offset = p.workspace_bytes;
    p.workspace_bytes += align256(bias_grad_partial_bytes(g));
    return p;
  }
  // (at most four channels and a narrow kernel matrix: the whole-matrix-per-block kernel below reads the input in place,
  // where this route writes a patch matrix first)
  if (bf16_mfma && pass == VCNN_PASS_BWD_FILTER && !(g.c <= 4 && g.k > 4 && filter_grad_few_cols_plan(g, &p.fcp)) &&
      bwd_filter_bf16_plan(g, &p.fb)) {
    p.path = PATH_FILTER_BF16;
    p.workspace_bytes = p.fb.dyt_bytes + p.fb.col_bytes + align256(p.fb.partial_bytes);
    p.bias_offset = p.workspace_bytes;
    p.workspace_bytes += align256(bias_grad_partial_bytes(g));
    return p;
  }
  if (pass == VCNN_PASS_FWD) {
    if (automatic && conv_taps_applies(g)) {
      p.path = PATH_TAPS;  // one map over many channels: the taps as rows of a 1 x 1 product, then a gather
      p.workspace_bytes = align256(conv_taps_fwd_bytes(g));
    } else if (allow_direct && g.k <= 4 && direct_fwd_geom(g, &p.dg) && direct_few_out_plan(&p.dg, &p.split, &p.partial_bytes)) {
      p.path = PATH_FEW_OUT;
      p.workspace_bytes = align256(p.partial_bytes);
    } else if (is_pointwise(g)) {
      p.path = PATH_POINTWISE;
    } else if (automatic && g.k > 4 && conv_small_applies(g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw)) {
      p.path = PATH_SMALL;  // a few hundred MFLOP: latency-bound, one tile per block and the contraction over its waves
    } else if (allow_direct && (g.c > 4 || g.k >= 32 || algo == VCNN_ALGO_IMPLICIT) &&
               conv_halo_plan(g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, &p.hp)) {
      p.path = PATH_HALO;
    } else if (allow_direct && g.c <= 4 && direct_fwd_geom(g, &p.dg) && direct_few_in_plan(&p.dg, &p.split)) {
      p.path = PATH_FEW_IN;
    } else {
      p.workspace_bytes = col_bytes(g);
    }
  } else if (pass == VCNN_PASS_BWD_DATA) {
    // the input gradient is a correlation of dy (k channels) with the flipped kernels into c maps
    if (algo == VCNN_ALGO_FOLD && !is_pointwise(g) && bwd_data_fold_plan(g, &p.fold)) {
      p.path = PATH_FOLD;
      p.workspace_bytes = align256(p.fold.partial_bytes);
    } else if (allow_direct && g.c <= 4 && direct_bwd_data_geom(g, &p.dg) &&
               direct_few_out_plan(&p.dg, &p.split, &p.partial_bytes)) {
      p.path = PATH_FEW_OUT;
      p.workspace_bytes = align256(p.partial_bytes);
    } else if (is_pointwise(g)) {
      p.path = PATH_POINTWISE;
    } else if (allow_direct && g.k <= 4 && g.c >= 64 && g.r - 1 - g.ph >= 0 && g.s - 1 - g.pw >= 0 &&
               conv_halo_plan(g.n, g.k, g.oh, g.ow, g.c, g.r, g.s, g.r - 1 - g.ph, g.s - 1 - g.pw, &p.hp)) {
      // few maps into many channels: the correlation's contraction is short (k*r*s) but it has many output maps,
      // which is matrix-core work; the flipped matrix lives in the workspace
      p.path = PATH_HALO;
      p.workspace_bytes = align256((size_t)g.M * g.K * sizeof(float));
    } else if (allow_direct && g.k <= 4 && direct_bwd_data_geom(g, &p.dg) && direct_few_in_plan(&p.dg, &p.split)) {
      p.path = PATH_FEW_IN;
    } else if (automatic && conv_small_bwd_applies(dtype, g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw)) {
      p.path = PATH_SMALL_BWD;  // transposed product and phi_c^{-1} fused on chip, no workspace
    } else if (automatic && g.c > 4 && g.r - 1 - g.ph >= 0 && g.s - 1 - g.pw >= 0 &&
               conv_small_applies(g.n, g.k, g.oh, g.ow, g.c, g.r, g.s, g.r - 1 - g.ph, g.s - 1 - g.pw)) {
      p.path = PATH_SMALL;  // the same latency-bound kernel on dy with the flipped matrix (kept in the workspace)
      p.workspace_bytes = align256((size_t)g.M * g.K * sizeof(float));
    } else if (allow_direct && g.r - 1 - g.ph >= 0 && g.s - 1 - g.pw >= 0 &&
               conv_halo_plan(g.n, g.k, g.oh, g.ow, g.c, g.r, g.s, g.r - 1 - g.ph, g.s - 1 - g.pw, &p.hp) &&
               (algo == VCNN_ALGO_IMPLICIT ||
                (halo_bwd_data_pays(g, p.hp) && !(automatic && bwd_data_fold_plan(g, &p.fold) && fold_beats_halo(g, p.hp, p.fold))))) {
      // correlation of dy (k channels) with the flipped kernels; the flipped matrix lives in the workspace
      p.path = PATH_HALO;
      p.workspace_bytes = align256((size_t)g.M * g.K * sizeof(float));
    } else if (automatic && bwd_data_fold_plan(g, &p.fold)) {
      // the paper's route (transposed product, then phi_c^{-1}) with the fold done per tile on chip
      p.path = PATH_FOLD;
      p.workspace_bytes = align256(p.fold.partial_bytes);
    } else {
      p.workspace_bytes = col_bytes(g);
    }
  } else {
    if (automatic && conv_taps_applies(g)) {
      p.path = PATH_TAPS;  // phi_c of the one-map gradient times the input, on the matrix cores
      p.workspace_bytes = conv_taps_filter_bytes(g, dtype);
    } else if (allow_direct && g.k <= 4 && direct_filter_grad_plan(g, &p.dg, &p.split, &p.partial_bytes)) {
      p.path = PATH_DIRECT_FILTER;
      p.workspace_bytes = align256(p.partial_bytes);
    } else if (automatic && g.k > 4 && filter_grad_few_cols_plan(g, &p.fcp)) {
      // narrow kernel matrix (the networks' first layers): every block computes the whole result for its pixels
      p.path = PATH_FEW_COLS_FILTER;
      p.workspace_bytes = align256(p.fcp.partial_bytes);
    } else if (allow_direct && (g.c > 4 || g.k >= 32 || algo == VCNN_ALGO_IMPLICIT) && conv_halo_filter_plan(g, &p.hfp)) {
      p.path = PATH_HALO_FILTER;
      p.workspace_bytes = align256(p.hfp.partial_bytes);
    } else if (automatic && is_pointwise(g) && g.k >= 32) {
      // the patch matrix of an unpadded 1 x 1 layer is the input itself: the product reads it in place
      p.path = PATH_POINTWISE;
      p.workspace_bytes = align256(bwd_filter_partial_bytes(g));
    } else if (allow_direct && direct_filter_grad_plan(g, &p.dg, &p.split, &p.partial_bytes)) {
      p.path = PATH_DIRECT_FILTER;
      p.workspace_bytes = align256(p.partial_bytes);
    } else {
      p.workspace_bytes = col_bytes(g) + align256(bwd_filter_partial_bytes(g));
    }
  }
  if (pass == VCNN_PASS_BWD_FILTER) {
    p.bias_offset = p.workspace_bytes;
    p.workspace_bytes += align256(bias_grad_partial_bytes(g));
  }
  return p;
}

static size_t workspace_need(const ConvGeom& g, int pass, int dtype) { return make_plan(g, pass, dtype).workspace_bytes; }

}  // namespace vcnn

using namespace vcnn;

extern "C" {

const char* vcnn_status_string(vcnn_status st) {
  switch (st) {
    case VCNN_OK: return "ok";
    case VCNN_ERR_NULL: return "null pointer";
    case VCNN_ERR_SHAPE: return "bad shape";
    case VCNN_ERR_WORKSPACE: return "bad workspace";
    case VCNN_ERR_UNSUPPORTED: return "unsupported";
    case VCNN_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* vcnn_last_error(void) { return g_err; }
int32_t vcnn_version(void) { return 100; }

vcnn_status vcnn_set_conv_algo(int32_t algo) {
  if (algo != VCNN_ALGO_AUTO && algo != VCNN_ALGO_EXPLICIT && algo != VCNN_ALGO_IMPLICIT && algo != VCNN_ALGO_FOLD &&
      algo != VCNN_ALGO_FFT && algo != VCNN_ALGO_SPLIT)
    return fail(VCNN_ERR_UNSUPPORTED, "unknown conv algorithm %d", algo);
  g_conv_algo.store(algo);
  return VCNN_OK;
}

vcnn_status vcnn_conv_out_shape(const vcnn_conv_desc* d, int32_t* oh, int32_t* ow) {
  if (!oh || !ow) return fail(VCNN_ERR_NULL, "conv_out_shape: NULL out-parameter");
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  *oh = g.oh, *ow = g.ow;
  return VCNN_OK;
}

vcnn_status vcnn_conv_workspace_bytes(const vcnn_conv_desc* d, int32_t pass, size_t* bytes) {
  if (!bytes) return fail(VCNN_ERR_NULL, "conv_workspace_bytes: NULL out-parameter");
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  if (pass < VCNN_PASS_FWD || pass > VCNN_PASS_BWD_DATA) return fail(VCNN_ERR_UNSUPPORTED, "unknown pass %d", pass);
  *bytes = workspace_need(g, pass, d->dtype);
  return VCNN_OK;
}

vcnn_status vcnn_im2col(const vcnn_conv_desc* d, const void* x, void* col, void* stream) {
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  if (!x || !col) return fail(VCNN_ERR_NULL, "im2col: NULL tensor");
  return launch_im2col(g, d->dtype, x, col, (hipStream_t)stream);
}

vcnn_status vcnn_col2im(const vcnn_conv_desc* d, const float* col, void* dx, void* stream) {
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  if (!col || !dx) return fail(VCNN_ERR_NULL, "col2im: NULL tensor");
  return launch_col2im(g, d->dtype, col, dx, (hipStream_t)stream);
}

static vcnn_status conv_fwd_linear(const vcnn_conv_desc* d, const ConvGeom& g, const void* x, const void* w,
                                   const float* bias, void* y, void* workspace, size_t workspace_bytes, void* stream);

vcnn_status vcnn_conv_fwd(const vcnn_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                          void* workspace, size_t workspace_bytes, void* stream) {
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  if (!x || !w || !y) return fail(VCNN_ERR_NULL, "conv_fwd: NULL tensor");
  if (vcnn_status s = conv_fwd_linear(d, g, x, w, bias, y, workspace, workspace_bytes, stream)) return s;
  // ReLU is applied inside the product's epilogue; the smooth sigma functions by one element-wise pass over y
  if (d->act == VCNN_ACT_TANH || d->act == VCNN_ACT_SIGMOID)
    return launch_smooth_act(d->act, d->dtype, (size_t)(g.M * g.N), y, nullptr, y, (hipStream_t)stream);
  return VCNN_OK;
}

static vcnn_status conv_fwd_linear(const vcnn_conv_desc* d, const ConvGeom& g, const void* x, const void* w,
                                   const float* bias, void* y, void* workspace, size_t workspace_bytes, void* stream) {
  const Plan plan = make_plan(g, VCNN_PASS_FWD, d->dtype);
  if (vcnn_status s = check_ws(workspace, workspace_bytes, plan.workspace_bytes, "conv_fwd")) return s;
  hipStream_t st = (hipStream_t)stream;
  const int relu = d->act == VCNN_ACT_RELU;
  const int dt = d->dtype;
  if (plan.path == PATH_TAPS) return launch_conv_taps_fwd(g, dt, x, w, bias, y, relu, (float*)workspace, st);
  if (plan.path == PATH_FEW_OUT)
    return launch_direct_few_out(plan.dg, dt, plan.split, x, w, bias, y, (float*)workspace, relu, st);
  if (plan.path == PATH_FEW_IN) return launch_direct_few_in(plan.dg, dt, plan.split, x, w, bias, y, relu, st);
  if (plan.path == PATH_SMALL)
    return launch_conv_small(dt, g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, x, w, bias, y, relu, st);
  if (plan.path == PATH_HALO)
    return launch_conv_halo(plan.hp, dt, g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, x, w, bias, y, relu, st);
  if (plan.path == PATH_HALO_BF16) {
    return launch_conv_halo_bf16(plan.hb, g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, x, w, g.K, (int64_t)g.r * g.s, 0,
                                 bias, y, relu, workspace, st);
  }
  if (plan.path == PATH_FFT) return launch_conv_fft(plan.fft, dt, g, x, w, bias, y, relu, workspace, st);
  if (plan.path == PATH_SPLIT)
    return launch_conv_split_fwd(plan.sp, g, (const float*)x, (const float*)w, bias, (float*)y, relu, workspace, st);
  // (its 16-byte reads of the kernel matrix need that alignment; a matrix placed otherwise takes the generic product)
  const bool pointwise_bf16 = plan.path == PATH_POINTWISE_BF16 && (reinterpret_cast<uintptr_t>(w) & 15) == 0;
  if (pointwise_bf16) return launch_pointwise_bf16(plan.pwb, g.n, g.k, g.c, (int)g.P, w, x, bias, y, relu, st);

  GemmArgs a{};
  a.A = w, a.C = y, a.bias = bias;
  a.in_dtype = dt, a.out_dtype = dt;
  a.M = (int)g.M, a.N = (int)g.N, a.K = (int)g.K;
  a.a_si = g.K, a.a_sk = 1;
  a.c_si = g.P, a.c_sj = 1, a.c_P = (int)g.P, a.c_simg = g.M * g.P;
  a.relu = relu;
  if (plan.path == PATH_POINTWISE || plan.path == PATH_POINTWISE_BF16) {
    // patch matrix == input: B(k, j) = x[n][k][p]
    a.B = x;
    a.b_sk = g.P, a.b_sj = 1, a.b_P = (int)g.P, a.b_simg = g.K * g.P;
  } else {
    if (vcnn_status s = launch_im2col(g, dt, x, workspace, st)) return s;
    a.B = workspace;
    a.b_sk = g.N, a.b_sj = 1, a.b_P = 0, a.b_simg = 0;
  }
  return launch_gemm_f32(a, st);
}

vcnn_status vcnn_conv_bwd_filter(const vcnn_conv_desc* d, const void* x, const void* dy, float* dw, float* dbias,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  if (!x || !dy || !dw) return fail(VCNN_ERR_NULL, "conv_bwd_filter: NULL tensor");
  const Plan plan = make_plan(g, VCNN_PASS_BWD_FILTER, d->dtype);
  if (vcnn_status s = check_ws(workspace, workspace_bytes, plan.workspace_bytes, "conv_bwd_filter")) return s;
  hipStream_t st = (hipStream_t)stream;
  const int dt = d->dtype;
  float* bias_partial = (float*)((char*)workspace + plan.bias_offset);
  if (plan.path == PATH_TAPS) {
    if (vcnn_status s = launch_conv_taps_filter(g, dt, x, dy, dw, workspace, st)) return s;
  } else if (plan.path == PATH_DIRECT_FILTER) {
    if (vcnn_status s = launch_direct_filter_grad(plan.dg, dt, plan.split, x, dy, dw, (float*)workspace, st)) return s;
  } else if (plan.path == PATH_FEW_COLS_FILTER) {
    if (vcnn_status s = launch_filter_grad_few_cols(plan.fcp, dt, g, x, dy, dw, dbias, (float*)workspace, st)) return s;
    if (plan.fcp.bias_column) return VCNN_OK;  // the bias gradient came out of the same product
  } else if (plan.path == PATH_SPLIT) {
    if (vcnn_status s = launch_conv_split_filter(plan.sp, g, (const float*)x, (const float*)dy, dw, workspace, st)) return s;
  } else if (plan.path == PATH_POINTWISE_BF16) {
    if (vcnn_status s = launch_pointwise_filter_bf16(plan.pwf, g, x, dy, dw, (float*)workspace, st)) return s;
  } else if (plan.path == PATH_HALO_FILTER_BF16) {
    if (vcnn_status s = launch_filter_grad_bf16(plan.hfb, g, x, dy, dw, workspace, st)) return s;
  } else if (plan.path == PATH_FILTER_BF16) {
    if (vcnn_status s = launch_bwd_filter_bf16(plan.fb, g, x, dy, dw, workspace, st)) return s;
  } else if (plan.path == PATH_HALO_FILTER) {
    if (vcnn_status s = launch_conv_halo_filter(plan.hfp, dt, g, x, dy, dw, dbias, (float*)workspace, st)) return s;
    if (plan.hfp.bias_column) return VCNN_OK;  // the bias gradient came out of the same product
  } else if (plan.path == PATH_POINTWISE) {
    if (vcnn_status s = launch_bwd_filter_gemm_f32(g, dt, dy, nullptr, x, dw, (float*)workspace, st)) return s;
  } else {
    float* partial = (float*)((char*)workspace + col_bytes(g));
    if (vcnn_status s = launch_im2col(g, dt, x, workspace, st)) return s;
    if (vcnn_status s = launch_bwd_filter_gemm_f32(g, dt, dy, workspace, nullptr, dw, partial, st)) return s;
  }
  if (dbias) return launch_bias_grad(g, dt, dy, dbias, bias_partial, st);
  return VCNN_OK;
}

// The input gradient, with sigma'(.) of the activation below (evaluated from x, that activation's forward output and this
// layer's input) folded in when act_below is not VCNN_ACT_NONE.  Routes whose last kernel writes one element of dx per
// thread (the fold's gather, the few-channel kernel) or already carry the factor (the plain products) apply it in
// that store; the matrix-core tile kernels do not - the reference values of a whole accumulator tile cost them a
// resident block per compute unit - and run the element-wise pass on dx in place afterwards.
static vcnn_status conv_bwd_data_impl(const vcnn_conv_desc* d, int act_below, const void* x, const void* w, const void* dy,
                                      void* dx, void* workspace, size_t workspace_bytes, void* stream, const char* who) {
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  if (act_below < VCNN_ACT_NONE || act_below > VCNN_ACT_SIGMOID) return fail(VCNN_ERR_UNSUPPORTED, "%s: unknown activation %d", who, act_below);
  if (!w || !dy || !dx || (act_below != VCNN_ACT_NONE && !x)) return fail(VCNN_ERR_NULL, "%s: NULL tensor", who);
  const Plan plan = make_plan(g, VCNN_PASS_BWD_DATA, d->dtype);
  if (vcnn_status s = check_ws(workspace, workspace_bytes, plan.workspace_bytes, who)) return s;
  hipStream_t st = (hipStream_t)stream;
  const int dt = d->dtype;
  const int da = act_below;
  const void* ref = da != VCNN_ACT_NONE ? x : nullptr;
  auto then_act = [&](vcnn_status s) {  // routes without the fused store
    if (s != VCNN_OK || da == VCNN_ACT_NONE) return s;
    return vcnn_act_bwd(da, dt, (size_t)g.n * g.c * g.h * g.w, x, dx, dx, stream);
  };
  if (plan.path == PATH_FEW_OUT)
    return then_act(launch_direct_few_out(plan.dg, dt, plan.split, dy, w, nullptr, dx, (float*)workspace, 0, st));
  if (plan.path == PATH_FEW_IN) return launch_direct_few_in(plan.dg, dt, plan.split, dy, w, nullptr, dx, 0, st, da, ref);
  if (plan.path == PATH_HALO_BF16) {
    // correlation of dy (k channels) with the flipped kernels into c maps: the re-ordering pass flips and transposes
    return then_act(launch_conv_halo_bf16(plan.hb, g.n, g.k, g.oh, g.ow, g.c, g.r, g.s, g.r - 1 - g.ph, g.s - 1 - g.pw, dy,
                                          w, (int64_t)g.r * g.s, g.K, 1, nullptr, dx, 0, workspace, st));
  }
  if (plan.path == PATH_POINTWISE_BF16) {
    // dx[n][c][p] = sum_m w[m][c] * dy[n][m][p]: the forward product on the transposed kernel matrix
    if (vcnn_status s = launch_flip_transpose(dt, w, workspace, g.k, g.c, 1, st)) return s;
    return then_act(launch_pointwise_bf16(plan.pwb, g.n, g.c, g.k, (int)g.P, workspace, dy, nullptr, dx, 0, st));
  }
  if (plan.path == PATH_SMALL_BWD)
    return then_act(launch_conv_small_bwd(g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.ph, g.pw, dy, w, dx, st));
  if (plan.path == PATH_SMALL) {
    if (vcnn_status s = launch_flip_transpose(dt, w, workspace, g.k, g.c, g.r * g.s, st)) return s;
    return then_act(launch_conv_small(dt, g.n, g.k, g.oh, g.ow, g.c, g.r, g.s, g.r - 1 - g.ph, g.s - 1 - g.pw, dy, workspace,
                                      nullptr, dx, 0, st));
  }
  if (plan.path == PATH_HALO) {
    if (vcnn_status s = launch_flip_transpose(dt, w, workspace, g.k, g.c, g.r * g.s, st)) return s;
    return then_act(launch_conv_halo(plan.hp, dt, g.n, g.k, g.oh, g.ow, g.c, g.r, g.s, g.r - 1 - g.ph, g.s - 1 - g.pw, dy,
                                     workspace, nullptr, dx, 0, st));
  }
  if (plan.path == PATH_FOLD) return launch_bwd_data_fold(plan.fold, dt, g, w, dy, dx, (float*)workspace, st, da, ref);
  // dcol[k][j] = sum_m W[m][k] * dY(m, j)
  GemmArgs a{};
  a.A = w, a.B = dy, a.bias = nullptr;
  a.in_dtype = dt;
  a.M = (int)g.K, a.N = (int)g.N, a.K = (int)g.M;
  a.a_si = 1, a.a_sk = g.K;
  a.b_sk = g.P, a.b_sj = 1, a.b_P = (int)g.P, a.b_simg = g.M * g.P;
  a.relu = 0;
  if (plan.path == PATH_POINTWISE) {
    // phi_c^{-1} is the identity per sample: store the product straight into dx[n][c][p].
    a.C = dx, a.out_dtype = dt;
    a.c_si = g.P, a.c_sj = 1, a.c_P = (int)g.P, a.c_simg = g.K * g.P;
    a.dact = da, a.dact_ref = ref;
    return launch_gemm_f32(a, st);
  }
  a.C = workspace, a.out_dtype = VCNN_F32;  // the patch-matrix gradient is kept in float
  a.c_si = g.N, a.c_sj = 1, a.c_P = 0, a.c_simg = 0;
  if (vcnn_status s = launch_gemm_f32(a, st)) return s;
  return then_act(launch_col2im(g, dt, (const float*)workspace, dx, st));
}

vcnn_status vcnn_conv_bwd_data(const vcnn_conv_desc* d, const void* w, const void* dy, void* dx, void* workspace,
                               size_t workspace_bytes, void* stream) {
  return conv_bwd_data_impl(d, VCNN_ACT_NONE, nullptr, w, dy, dx, workspace, workspace_bytes, stream, "conv_bwd_data");
}

vcnn_status vcnn_conv_bwd_data_act(const vcnn_conv_desc* d, int32_t act_below, const void* x, const void* w, const void* dy,
                                   void* dx, void* workspace, size_t workspace_bytes, void* stream) {
  return conv_bwd_data_impl(d, act_below, x, w, dy, dx, workspace, workspace_bytes, stream, "conv_bwd_data_act");
}

// ---- the kernel-gradient pass for callers that cannot allocate ----------------------------------------
// The partial sums of the split contraction (and of the bias gradient) live in a fixed array of the code object
// instead of a caller workspace.  Every GPU the library runs on holds its own copy of the array, at its own address,
// until the process ends; host code never uses the array's name as an address, only what hipGetSymbolAddress
// returned for the device that is current.
static constexpr size_t kScratchBytes = (size_t)32 << 20;
static constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static vcnn_status scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(VCNN_ERR_HIP, "conv_bwd_filter_noalloc: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(VCNN_ERR_UNSUPPORTED, "conv_bwd_filter_noalloc: device index %d", dev);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {  // once per device (a second thread racing here looks the same address up again)
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return fail(VCNN_ERR_HIP, "conv_bwd_filter_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return VCNN_OK;
}

size_t vcnn_conv_bwd_filter_noalloc_limit(void) { return kScratchBytes; }

vcnn_status vcnn_conv_bwd_filter_noalloc(const vcnn_conv_desc* d, const void* x, const void* dy, float* dw,
                                         float* dbias, void* stream) {
  ConvGeom g;
  if (vcnn_status s = make_geom(d, &g)) return s;
  if (!x || !dy || !dw) return fail(VCNN_ERR_NULL, "conv_bwd_filter_noalloc: NULL tensor");
  const size_t need = workspace_need(g, VCNN_PASS_BWD_FILTER, d->dtype);
  if (need > kScratchBytes)
    return fail(VCNN_ERR_WORKSPACE,
                "conv_bwd_filter_noalloc: this layer needs %zu bytes of scratch memory, the built-in array holds %zu; "
                "use vcnn_conv_bwd_filter with a workspace", need, kScratchBytes);
  void* ws = nullptr;
  if (vcnn_status s = scratch_of_current_device(&ws)) return s;
  // nothing in the pass reads scratch memory it has not written in the same call, so nothing needs clearing
  return vcnn_conv_bwd_filter(d, x, dy, dw, dbias, ws, kScratchBytes, stream);
}

static vcnn_status check_pool(const vcnn_pool_desc* d, int* oh, int* ow) {
  if (!d) return fail(VCNN_ERR_NULL, "pool descriptor is NULL");
  if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->win_h <= 0 || d->win_w <= 0 || d->stride_h <= 0 ||
      d->stride_w <= 0)
    return fail(VCNN_ERR_SHAPE, "pool: non-positive dimension");
  if (d->win_h > d->h || d->win_w > d->w)
    return fail(VCNN_ERR_SHAPE, "pool: window %dx%d larger than input %dx%d", d->win_h, d->win_w, d->h, d->w);
  if ((int64_t)d->h * d->w > 0x7fffffffLL) return fail(VCNN_ERR_UNSUPPORTED, "pool: plane too large for int32 indices");
  if (vcnn_status s = check_dtype(d->dtype, "pool")) return s;
  if (d->mode != VCNN_POOL_MAX && d->mode != VCNN_POOL_AVG) return fail(VCNN_ERR_UNSUPPORTED, "pool: unknown mode %d", d->mode);
  *oh = (d->h - d->win_h) / d->stride_h + 1;
  *ow = (d->w - d->win_w) / d->stride_w + 1;
  return VCNN_OK;
}

vcnn_status vcnn_pool_out_shape(const vcnn_pool_desc* d, int32_t* oh, int32_t* ow) {
  if (!oh || !ow) return fail(VCNN_ERR_NULL, "pool_out_shape: NULL out-parameter");
  int a, b;
  if (vcnn_status s = check_pool(d, &a, &b)) return s;
  *oh = a, *ow = b;
  return VCNN_OK;
}

static bool known_act(int32_t act) {
  return act == VCNN_ACT_NONE || act == VCNN_ACT_RELU || act == VCNN_ACT_TANH || act == VCNN_ACT_SIGMOID;
}

vcnn_status vcnn_pool_layer_fwd(const vcnn_pool_desc* d, int32_t act, const void* x, const float* bias, void* y,
                                int32_t* argmax, void* stream) {
  int oh, ow;
  if (vcnn_status s = check_pool(d, &oh, &ow)) return s;
  if (!known_act(act)) return fail(VCNN_ERR_UNSUPPORTED, "pool_layer_fwd: activation %d is not built", act);
  if (!x || !y || (!argmax && d->mode == VCNN_POOL_MAX)) return fail(VCNN_ERR_NULL, "pool_fwd: NULL tensor");
  if (d->mode == VCNN_POOL_AVG) return launch_avgpool(*d, oh, ow, x, y, false, bias, act, (hipStream_t)stream);
  return launch_pool_fwd(*d, oh, ow, x, y, argmax, bias, act, (hipStream_t)stream);
}

vcnn_status vcnn_pool_fwd(const vcnn_pool_desc* d, const void* x, void* y, int32_t* argmax, void* stream) {
  return vcnn_pool_layer_fwd(d, VCNN_ACT_NONE, x, nullptr, y, argmax, stream);
}

// the pooled maps as the (n, M = maps, P = pixels per map) view the bias-gradient reduction takes
static ConvGeom pooled_geom(const vcnn_pool_desc& d, int oh, int ow) {
  ConvGeom g{};
  g.n = d.n, g.M = d.c, g.P = (int64_t)oh * ow;
  return g;
}

static size_t pool_delta_bytes(const vcnn_pool_desc& d, int oh, int ow) {
  return align256((size_t)d.n * d.c * oh * ow * (d.dtype == VCNN_BF16 ? 2 : 4));
}

vcnn_status vcnn_pool_layer_workspace_bytes(const vcnn_pool_desc* d, size_t* bytes) {
  if (!bytes) return fail(VCNN_ERR_NULL, "pool_layer_workspace_bytes: NULL out-parameter");
  int oh, ow;
  if (vcnn_status s = check_pool(d, &oh, &ow)) return s;
  *bytes = pool_delta_bytes(*d, oh, ow) + align256(bias_grad_partial_bytes(pooled_geom(*d, oh, ow)));
  return VCNN_OK;
}

vcnn_status vcnn_pool_layer_bwd(const vcnn_pool_desc* d, int32_t act, const void* y, const void* dy,
                                const int32_t* argmax, float* dbias, void* dx, void* workspace, size_t workspace_bytes,
                                void* stream) {
  int oh, ow;
  if (vcnn_status s = check_pool(d, &oh, &ow)) return s;
  if (!known_act(act)) return fail(VCNN_ERR_UNSUPPORTED, "pool_layer_bwd: activation %d is not built", act);
  if (!dy || !dx || (act != VCNN_ACT_NONE && !y) || (!argmax && d->mode == VCNN_POOL_MAX))
    return fail(VCNN_ERR_NULL, "pool_layer_bwd: NULL tensor");
  size_t need = 0;
  (void)vcnn_pool_layer_workspace_bytes(d, &need);
  if (act == VCNN_ACT_NONE && !dbias) need = 0;
  if (need && (!workspace || workspace_bytes < need))
    return fail(VCNN_ERR_WORKSPACE, "pool_layer_bwd: workspace has %zu bytes, needs %zu", workspace_bytes, need);
  // delta = dy * sigma'(.) from y; then the two gradients read delta
  const void* delta = dy;
  if (act != VCNN_ACT_NONE) {
    if (vcnn_status s = vcnn_act_bwd(act, d->dtype, (size_t)d->n * d->c * oh * ow, y, dy, workspace, stream)) return s;
    delta = workspace;
  }
  if (dbias) {
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + pool_delta_bytes(*d, oh, ow));
    if (vcnn_status s = launch_bias_grad(pooled_geom(*d, oh, ow), d->dtype, delta, dbias, partial, (hipStream_t)stream))
      return s;
  }
  return vcnn_pool_bwd(d, delta, argmax, dx, stream);
}

vcnn_status vcnn_pool_bwd(const vcnn_pool_desc* d, const void* dy, const int32_t* argmax, void* dx, void* stream) {
  int oh, ow;
  if (vcnn_status s = check_pool(d, &oh, &ow)) return s;
  if (!dy || !dx || (!argmax && d->mode == VCNN_POOL_MAX)) return fail(VCNN_ERR_NULL, "pool_bwd: NULL tensor");
  if (d->mode == VCNN_POOL_AVG) return launch_avgpool(*d, oh, ow, dy, dx, true, nullptr, VCNN_ACT_NONE, (hipStream_t)stream);
  return launch_pool_bwd(*d, oh, ow, dy, argmax, dx, VCNN_ACT_NONE, nullptr, (hipStream_t)stream);
}

vcnn_status vcnn_pool_bwd_act(const vcnn_pool_desc* d, int32_t act_below, const void* x, const void* dy,
                              const int32_t* argmax, void* dx, void* stream) {
  if (act_below == VCNN_ACT_NONE) return vcnn_pool_bwd(d, dy, argmax, dx, stream);
  if (act_below != VCNN_ACT_RELU && act_below != VCNN_ACT_TANH && act_below != VCNN_ACT_SIGMOID)
    return fail(VCNN_ERR_UNSUPPORTED, "pool_bwd_act: activation %d is not built", act_below);
  int oh, ow;
  if (vcnn_status s = check_pool(d, &oh, &ow)) return s;
  if (!x || !dy || !dx || (!argmax && d->mode == VCNN_POOL_MAX)) return fail(VCNN_ERR_NULL, "pool_bwd_act: NULL tensor");
  if (d->mode == VCNN_POOL_AVG) {  // the transpose of the mean, then the derivative in place
    if (vcnn_status s = launch_avgpool(*d, oh, ow, dy, dx, true, nullptr, VCNN_ACT_NONE, (hipStream_t)stream)) return s;
    return vcnn_act_bwd(act_below, d->dtype, (size_t)d->n * d->c * d->h * d->w, x, dx, dx, stream);
  }
  return launch_pool_bwd(*d, oh, ow, dy, argmax, dx, act_below, x, (hipStream_t)stream);
}

vcnn_status vcnn_act_fwd(int32_t act, int32_t dtype, size_t count, const void* x, void* y, void* stream) {
  if (act != VCNN_ACT_RELU && act != VCNN_ACT_TANH && act != VCNN_ACT_SIGMOID)
    return fail(VCNN_ERR_UNSUPPORTED, "act_fwd: activation %d is not built", act);
  if (vcnn_status s = check_dtype(dtype, "act_fwd")) return s;
  if (count == 0) return VCNN_OK;
  if (!x || !y) return fail(VCNN_ERR_NULL, "act_fwd: NULL tensor");
  if (act != VCNN_ACT_RELU) return launch_smooth_act(act, dtype, count, x, nullptr, y, (hipStream_t)stream);
  return launch_relu_fwd(dtype, count, x, y, (hipStream_t)stream);
}

vcnn_status vcnn_act_bwd(int32_t act, int32_t dtype, size_t count, const void* ref, const void* dy, void* dx,
                         void* stream) {
  if (act != VCNN_ACT_RELU && act != VCNN_ACT_TANH && act != VCNN_ACT_SIGMOID)
    return fail(VCNN_ERR_UNSUPPORTED, "act_bwd: activation %d is not built", act);
  if (vcnn_status s = check_dtype(dtype, "act_bwd")) return s;
  if (count == 0) return VCNN_OK;
  if (!ref || !dy || !dx) return fail(VCNN_ERR_NULL, "act_bwd: NULL tensor");
  if (act != VCNN_ACT_RELU) return launch_smooth_act(act, dtype, count, ref, dy, dx, (hipStream_t)stream);
  return launch_relu_bwd(dtype, count, ref, dy, dx, (hipStream_t)stream);
}

static vcnn_status check_fc(int32_t batch, int32_t in_f, int32_t out_f) {
  if (batch <= 0 || in_f <= 0 || out_f <= 0)
    return fail(VCNN_ERR_SHAPE, "fc: non-positive dimension (batch=%d in=%d out=%d)", batch, in_f, out_f);
  return VCNN_OK;
}

vcnn_status vcnn_fc_fwd(int32_t dtype, int32_t batch, int32_t in_f, int32_t out_f, int32_t act, const void* x,
                        const void* w, const float* bias, void* y, void* stream) {
  if (vcnn_status s = check_fc(batch, in_f, out_f)) return s;
  if (act < VCNN_ACT_NONE || act > VCNN_ACT_SIGMOID) return fail(VCNN_ERR_UNSUPPORTED, "fc_fwd: unknown activation %d", act);
  if (vcnn_status s = check_dtype(dtype, "fc_fwd")) return s;
  if (!x || !w || !y) return fail(VCNN_ERR_NULL, "fc_fwd: NULL tensor");
  // C(i = o, j = b) = sum_k W[o][k] * X[b][k], stored at y[b*O + o]
  GemmArgs a{};
  a.A = w, a.B = x, a.C = y, a.bias = bias;
  a.in_dtype = dtype, a.out_dtype = dtype;
  a.M = out_f, a.N = batch, a.K = in_f;
  a.a_si = in_f, a.a_sk = 1;
  a.b_sk = 1, a.b_sj = in_f, a.b_P = 0;
  a.c_si = 1, a.c_sj = out_f, a.c_P = 0;
  a.relu = act == VCNN_ACT_RELU;
  if (vcnn_status s = launch_gemm_f32(a, (hipStream_t)stream)) return s;
  if (act == VCNN_ACT_TANH || act == VCNN_ACT_SIGMOID)
    return launch_smooth_act(act, dtype, (size_t)batch * out_f, y, nullptr, y, (hipStream_t)stream);
  return VCNN_OK;
}

static vcnn_status fc_bwd_impl(int32_t dtype, int32_t batch, int32_t in_f, int32_t out_f, int32_t act_below,
                               const void* x, const void* w, const void* dy, float* dw, float* dbias, void* dx,
                               void* stream) {
  if (vcnn_status s = check_fc(batch, in_f, out_f)) return s;
  if (vcnn_status s = check_dtype(dtype, "fc_bwd")) return s;
  if (act_below != VCNN_ACT_NONE && act_below != VCNN_ACT_RELU && act_below != VCNN_ACT_TANH &&
      act_below != VCNN_ACT_SIGMOID)
    return fail(VCNN_ERR_UNSUPPORTED, "fc_bwd: activation %d is not built", act_below);
  if (!dy || ((dw || (dx && act_below)) && !x) || (dx && !w)) return fail(VCNN_ERR_NULL, "fc_bwd: NULL tensor");
  hipStream_t st = (hipStream_t)stream;
  GemmArgs gw{}, gx{};
  // dW(i = o, j = i_) = sum_b dY[b][o] * X[b][i_]
  gw.A = dy, gw.B = x, gw.C = dw;
  gw.in_dtype = dtype, gw.out_dtype = VCNN_F32;
  gw.M = out_f, gw.N = in_f, gw.K = batch;
  gw.a_si = 1, gw.a_sk = out_f;
  gw.b_sk = in_f, gw.b_sj = 1, gw.b_P = 0;
  gw.c_si = in_f, gw.c_sj = 1, gw.c_P = 0;
  // dX(i = b, j = i_) = sum_o dY[b][o] * W[o][i_]
  gx.A = dy, gx.B = w, gx.C = dx;
  gx.in_dtype = dtype, gx.out_dtype = dtype;
  gx.M = batch, gx.N = in_f, gx.K = out_f;
  gx.a_si = out_f, gx.a_sk = 1;
  gx.b_sk = in_f, gx.b_sj = 1, gx.b_P = 0;
  gx.c_si = in_f, gx.c_sj = 1, gx.c_P = 0;
  gx.dact = act_below, gx.dact_ref = act_below ? x : nullptr;
  // the small-product kernel takes the bias gradient along as the weight gradient's column of ones
  gw.row_sums = dbias;
  if (dw && gemm_is_small(gw)) dbias = nullptr;
  else gw.row_sums = nullptr;
  if (dw && dx && gemm_is_small(gw) && gemm_is_small(gx)) {
    if (vcnn_status s = launch_fc_bwd_small(gw, gx, st)) return s;
    dw = nullptr, dx = nullptr;
  }
  if (dw)
    if (vcnn_status s = launch_gemm_f32(gw, st)) return s;
  if (dbias)
    if (vcnn_status s = launch_col_sum(dtype, batch, out_f, dy, dbias, st)) return s;
  if (dx)
    if (vcnn_status s = launch_gemm_f32(gx, st)) return s;
  return VCNN_OK;
}

vcnn_status vcnn_fc_bwd(int32_t dtype, int32_t batch, int32_t in_f, int32_t out_f, const void* x, const void* w,
                        const void* dy, float* dw, float* dbias, void* dx, void* stream) {
  return fc_bwd_impl(dtype, batch, in_f, out_f, VCNN_ACT_NONE, x, w, dy, dw, dbias, dx, stream);
}

vcnn_status vcnn_fc_bwd_act(int32_t dtype, int32_t batch, int32_t in_f, int32_t out_f, int32_t act_below,
                            const void* x, const void* w, const void* dy, float* dw, float* dbias, void* dx,
                            void* stream) {
  return fc_bwd_impl(dtype, batch, in_f, out_f, act_below, x, w, dy, dw, dbias, dx, stream);
}

vcnn_status vcnn_softmax_loss(int32_t batch, int32_t classes, const float* logits, const int32_t* labels, float* loss,
                              float* dlogits, void* stream) {
  if (batch <= 0 || classes <= 0) return fail(VCNN_ERR_SHAPE, "softmax_loss: non-positive dimension");
  if (!logits || !labels || !loss) return fail(VCNN_ERR_NULL, "softmax_loss: NULL tensor");
  return launch_softmax_loss_f32(batch, classes, logits, labels, loss, dlogits, (hipStream_t)stream);
}

vcnn_status vcnn_l2_loss(int32_t dtype, size_t count, int32_t batch, const void* y, const float* target, float* loss,
                         void* dy, void* stream) {
  if (batch <= 0 || count == 0) return fail(VCNN_ERR_SHAPE, "l2_loss: empty tensor");
  if (vcnn_status s = check_dtype(dtype, "l2_loss")) return s;
  if (!y || !target) return fail(VCNN_ERR_NULL, "l2_loss: NULL tensor");
  return launch_l2_loss(dtype, count, batch, y, target, loss, dy, (hipStream_t)stream);
}

vcnn_status vcnn_sgd_update(size_t count, float lr, float* w, const float* dw, void* stream) {
  if (count == 0) return VCNN_OK;
  if (!w || !dw) return fail(VCNN_ERR_NULL, "sgd_update: NULL tensor");
  return launch_sgd_f32(count, lr, w, dw, (hipStream_t)stream);
}

vcnn_status vcnn_sgd_update_multi(int32_t tensors, const size_t* counts, float* const* w, const float* const* dw,
                                  void* const* w_bf16, float lr, void* stream) {
  if (tensors < 0) return fail(VCNN_ERR_SHAPE, "sgd_update_multi: negative tensor count");
  if (tensors == 0) return VCNN_OK;
  if (!counts || !w || !dw) return fail(VCNN_ERR_NULL, "sgd_update_multi: NULL argument array");
  const uint64_t max_blocks = 0x7fffffffULL;  // of one launch
  for (int t = 0; t < tensors; ++t) {  // all checks before the first launch: an error leaves every tensor as it was
    if (counts[t] > 0 && (!w[t] || !dw[t])) return fail(VCNN_ERR_NULL, "sgd_update_multi: NULL tensor %d", t);
    if ((counts[t] + 255) / 256 > max_blocks) return fail(VCNN_ERR_SHAPE, "sgd_update_multi: tensor %d has too many elements", t);
  }
  // batches of up to kSgdBatch non-empty tensors and max_blocks blocks; t carries on where the previous batch stopped
  for (int t = 0; t < tensors;) {
    SgdBatch a{};
    a.lr = lr;
    uint64_t blocks = 0;
    for (; t < tensors && a.tensors < kSgdBatch; ++t) {
      if (counts[t] == 0) continue;
      const uint64_t more = (counts[t] + 255) / 256;
      if (blocks + more > max_blocks) break;  // this tensor opens the next batch
      const int k = a.tensors++;
      a.w[k] = w[t], a.dw[k] = dw[t], a.w16[k] = w_bf16 ? w_bf16[t] : nullptr, a.count[k] = counts[t];
      a.first[k] = (unsigned)blocks;
      blocks += more;
    }
    if (a.tensors == 0) break;
    a.first[a.tensors] = (unsigned)blocks;
    if (vcnn_status s = launch_sgd_multi(a, (hipStream_t)stream)) return s;
  }
  return VCNN_OK;
}

vcnn_status vcnn_f32_to_bf16(size_t count, const float* src, void* dst, void* stream) {
  if (count == 0) return VCNN_OK;
  if (!src || !dst) return fail(VCNN_ERR_NULL, "f32_to_bf16: NULL tensor");
  return launch_f32_to_bf16(count, src, (uint16_t*)dst, (hipStream_t)stream);
}

vcnn_status vcnn_bf16_to_f32(size_t count, const void* src, float* dst, void* stream) {
  if (count == 0) return VCNN_OK;
  if (!src || !dst) return fail(VCNN_ERR_NULL, "bf16_to_f32: NULL tensor");
  return launch_bf16_to_f32(count, (const uint16_t*)src, dst, (hipStream_t)stream);
}

}  // extern "C"
