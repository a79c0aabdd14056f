// Input gradient on the paper's own route - the transposed product dcol = W^T * dY followed by the
// many-to-one operator phi_c^{-1} (back-propagation paragraph of "Vectorizing Convolution") - without the
// patch-matrix gradient ever reaching memory.
//
// The product is the plain dense one: rows i = (c, r, s) of the kernel matrix, columns j = (oh, ow) of one
// sample, contraction over the output maps, exactly 2*M*K*N flop (nothing multiplies a zero border, which the
// gather form - a fully padded correlation - does for 'valid' layers).  A block owns a BM x BN tile of dcol of
// one sample.  When its accumulators are complete it folds them on chip: entry (i, j) belongs to input pixel
// (c, oh + r - pad_h, ow + s - pad_w), and all pixels a tile can touch form a small region (the tile's channels x
// a few input rows x the row width) held in LDS.  Every half-wave adds into a private copy of that region - lanes
// of one half-wave hold one row i and distinct columns, hence distinct pixels, and a wave's LDS accesses execute
// in program order - and the copies are then added in a fixed order, so no atomic is involved and the result is
// bit-identical from run to run.  The region (a few KB instead of BM x BN floats) goes to the workspace; a second
// small kernel adds, for every input pixel, the regions that cover it in ascending tile order.
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "common.h"
#include "elem.h"
#include "mma_core.h"

namespace vcnn {

static constexpr int kThreads = 256;
static constexpr int kFoldBM = 128, kFoldBN = 128, kFoldBK = 16;
static constexpr int kCopies = 8;  // 4 waves x 2 half-waves
static constexpr int kPatchI = 8, kPatchJ = 16;

struct FoldArgs {
  const void* w;    // [m][K]           kernel matrix as stored (row = output map), element type T
  const void* dy;   // [n][m][P]        element type T
  float* partial;   // [n][tiles_i][tiles_j][rsz]
  void* dx;         // [n][c][h][wd]    element type T (second pass)
  int n, c, h, wd, m, r, s, ph, pw, oh, ow, P, K;
  int tiles_i, tiles_j;
  int rsz;          // floats per region slot
  int wreg;         // region row width = ow + s - 1 (input columns -pw .. ow + s - 2 - pw)
  int dact;         // second pass, VCNN_ACT_*: dx is multiplied by sigma'(.) evaluated from dact_ref (shape and type of dx)
  const void* dact_ref;
};

// Geometry of the region tile (it, jt) folds into: channels c_lo .. c_lo + nch - 1, region rows = input rows
// h_lo .. h_lo + nrows - 1 (may stick out of the image; those rows are never read back).
struct FoldRegion {
  int c_lo, nch, r_lo, r_hi, h_lo, nrows, oh_first;
};
__host__ __device__ inline FoldRegion fold_region(int it, int jt, int K, int P, int RS, int S, int R, int OW, int ph) {
  FoldRegion g;
  const int i_first = it * kFoldBM, i_last = (it * kFoldBM + kFoldBM < K ? it * kFoldBM + kFoldBM : K) - 1;
  const int c_hi = i_last / RS;
  g.c_lo = i_first / RS;
  g.nch = c_hi - g.c_lo + 1;
  g.r_lo = 0, g.r_hi = R - 1;
  if (g.nch == 1) g.r_lo = (i_first - g.c_lo * RS) / S, g.r_hi = (i_last - g.c_lo * RS) / S;
  const int p_first = jt * kFoldBN, p_last = (jt * kFoldBN + kFoldBN < P ? jt * kFoldBN + kFoldBN : P) - 1;
  g.oh_first = p_first / OW;
  const int oh_last = p_last / OW;
  g.h_lo = g.oh_first + g.r_lo - ph;
  g.nrows = (oh_last - g.oh_first) + (g.r_hi - g.r_lo) + 1;
  return g;
}

template <bool A_VEC, bool B_VEC, bool MI_INDEP, typename T>
__global__ __launch_bounds__(kThreads, 4) void bwd_data_fold_kernel(FoldArgs a) {
  constexpr int BM = kFoldBM, BN = kFoldBN, BK = kFoldBK, WM = 64, WN = 64, TM = 2, TN = 2;
  using LA = LdsTile<BM, BK, false>;
  using LB = LdsTile<BN, BK, false>;
  using SA = Stager<BM, BK, kThreads, false, A_VEC>;
  using SB = Stager<BN, BK, kThreads, false, B_VEC>;
  extern __shared__ float4 smem4[];
  float* smem = reinterpret_cast<float*>(smem4);
  float* const As0 = smem;
  float* const Bs0 = smem + 2 * LA::SIZE;

  const T* gA = static_cast<const T*>(a.w);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // Block order.  Consecutive block ids go round-robin to the 8 XCDs, each with its own L2: give every XCD a
  // contiguous run of the order below.  That order walks the tile grid (row tiles x all samples' column tiles) in
  // patches of kPatchI x kPatchJ tiles - about what one XCD holds resident at once -, so the blocks resident
  // together share kPatchI panels of the kernel matrix and kPatchJ panels of dy in L2 instead of sweeping one of the
  // operands whole.
  int it, tj;
  {
    const int total = gridDim.x;
    const int per = total / 8;
    const int t = (int)blockIdx.x < per * 8 ? ((int)blockIdx.x % 8) * per + (int)blockIdx.x / 8 : (int)blockIdx.x;
    const int TI = a.tiles_i, TJ = a.n * a.tiles_j;
    const int pj = t / (TI * kPatchJ);
    const int rem = t - pj * (TI * kPatchJ);
    const int wj = min(kPatchJ, TJ - pj * kPatchJ);
    const int pi = rem / (kPatchI * wj);
    const int rem2 = rem - pi * (kPatchI * wj);
    const int hi = min(kPatchI, TI - pi * kPatchI);
    const int jl = rem2 / hi;
    it = pi * kPatchI + (rem2 - jl * hi);
    tj = pj * kPatchJ + jl;
  }
  const int n = tj / a.tiles_j, jt = tj - n * a.tiles_j;
  const int i0 = it * BM, j0 = jt * BN;
  const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
  const T* gB = static_cast<const T*>(a.dy) + (int64_t)n * a.m * a.P;

  SA sa;
  SB sb;
  sa.init(tid);
  sb.init(tid);
  // A(i, k) = w[k][i] (contiguous along i), B(k, j) = dy[n][k][j] (contiguous along j); slots outside the matrix
  // read a valid address and are zeroed when the slab is written to LDS
  // A_VEC: four rows per 16-byte load at dword alignment (float) or 8-byte load (bf16: K a multiple of 4).  The
  // matrix's last group may hold fewer than four rows: the load is moved back to the last four (K >= 4) and the
  // wanted ones are shifted down, zeros behind them.
  const bool a_ok = i0 + sa.c < a.K;
  const int a_i = a_ok ? (A_VEC ? min(i0 + sa.c, a.K - 4) : i0 + sa.c) : 0;
  const int a_d = a_ok ? i0 + sa.c - a_i : 0;
  const bool b_ok = j0 + sb.c < a.P;
  // B_VEC (float only): four pixels per 16-byte load at dword alignment; the sample's last group may end early - its
  // load is moved back to the last four pixels (P >= 4) and the wanted ones are shifted down, zeros behind them
  const int b_j = b_ok ? (B_VEC ? min(j0 + sb.c, a.P - 4) : j0 + sb.c) : 0;
  const int b_d = b_ok ? j0 + sb.c - b_j : 0;
  auto fetch = [&](int k0) {
#pragma unroll
    for (int e = 0; e < SA::SLOTS; ++e) {
      const int k = k0 + sa.line(e);
      sa.ok[e] = a_ok && k < a.m;
      const T* src = gA + (int64_t)min(k, a.m - 1) * a.K + a_i;
      if constexpr (A_VEC) {
        float4 t;
        if constexpr (std::is_same<T, float>::value) t = ld4_dword_aligned(src);
        else t = ld4(src);
        sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
        if (a_d > 0) {
          sa.v[e][0] = a_d == 1 ? t.y : (a_d == 2 ? t.z : t.w);
          sa.v[e][1] = a_d == 1 ? t.z : (a_d == 2 ? t.w : 0.f);
          sa.v[e][2] = a_d == 1 ? t.w : 0.f;
          sa.v[e][3] = 0.f;
        }
      } else {
        sa.v[e][0] = ld(src);
      }
    }
#pragma unroll
    for (int e = 0; e < SB::SLOTS; ++e) {
      const int k = k0 + sb.line(e);
      sb.ok[e] = b_ok && k < a.m;
      const T* src = gB + (int64_t)min(k, a.m - 1) * a.P + b_j;
      if constexpr (B_VEC && std::is_same<T, float>::value) {
        const float4 t = ld4_dword_aligned(src);
        sb.v[e][0] = t.x, sb.v[e][1] = t.y, sb.v[e][2] = t.z, sb.v[e][3] = t.w;
        if (b_d > 0) {
          sb.v[e][0] = b_d == 1 ? t.y : (b_d == 2 ? t.z : t.w);
          sb.v[e][1] = b_d == 1 ? t.z : (b_d == 2 ? t.w : 0.f);
          sb.v[e][2] = b_d == 1 ? t.w : 0.f;
          sb.v[e][3] = 0.f;
        }
      } else {
        sb.v[e][0] = ld(src);
      }
    }
  };

  f32x16 acc[TM][TN];
  zero_acc<TM, TN>(acc);
  const int ktiles = (a.m + BK - 1) / BK;
  fetch(0);
  sa.store(As0);
  sb.store(Bs0);
  __syncthreads();
  for (int kt = 0; kt < ktiles; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < ktiles) fetch((kt + 1) * BK);
    mma_slab<BM, BN, BK, TM, TN, false, false>(As0 + cur * LA::SIZE, Bs0 + cur * LB::SIZE, wm0, wn0, lane, acc);
    if (kt + 1 < ktiles) {
      sa.store(As0 + (cur ^ 1) * LA::SIZE);
      sb.store(Bs0 + (cur ^ 1) * LB::SIZE);
    }
    __syncthreads();
  }

  // ---- phi_c^{-1} of the tile, on chip ----------------------------------------------------------------------
  const int RS = a.r * a.s;
  const FoldRegion g = fold_region(it, jt, a.K, a.P, RS, a.s, a.r, a.ow, a.ph);
  float* const reg0 = smem;  // kCopies x rsz floats, over the operand slabs (all waves are past the last barrier)
  int* const rowtab = reinterpret_cast<int*>(reg0 + kCopies * a.rsz);  // [BM] region offset of the tile's rows
  for (int e = tid; e < kCopies * a.rsz; e += kThreads) reg0[e] = 0.f;
  if (tid < BM) {  // row i = (channel, kernel row, kernel column) -> offset of its tap inside the region; -1 beyond the matrix
    const int i = i0 + tid;
    const int ci = i / RS;
    const int t = i - ci * RS;
    const int r = t / a.s;
    rowtab[tid] = i < a.K ? (ci - g.c_lo) * (g.nrows * a.wreg) + (r - g.r_lo) * a.wreg + (t - r * a.s) : -1;
  }
  __syncthreads();
  const int l32 = lane & 31, half = lane >> 5;
  float* const mine = reg0 + (wave * 2 + half) * a.rsz;
  const int plane = g.nrows * a.wreg;
  // region offset of this lane's two columns (pixels), relative to the tap (r_lo, s = 0) of channel c_lo
  int col_off[TN];
  bool col_ok[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = j0 + wn0 + ni * 32 + l32;
    col_ok[ni] = p < a.P;
    const int pc = col_ok[ni] ? p : j0;
    const int oh = pc / a.ow;
    col_off[ni] = (oh - g.oh_first) * a.wreg + (pc - oh * a.ow);
  }
  // Neighbouring taps of one lane are neighbouring pixels of its neighbour lanes, so an add must see the adds of
  // the steps before it: steps run strictly in program order (a wave's LDS accesses do).  Inside one step the
  // addresses are provably distinct - a row's two column blocks are different pixels; rows 32 apart differ by a tap
  // offset no pair of the wave's 64 pixels has (MI_INDEP, checked on the host) - so a step reads all its entries,
  // adds, and writes them: one LDS round trip per step.
  if (MI_INDEP) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      int off[TM];
      float v[TM][TN];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi) off[mi] = rowtab[wm0 + mi * 32 + acc_row(q, lane)];  // -1: row beyond the matrix
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) v[mi][ni] = mine[max(off[mi], 0) + col_off[ni]];
#pragma unroll
      for (int mi = 0; mi < TM; ++mi)
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
          if (off[mi] >= 0 && col_ok[ni]) mine[off[mi] + col_off[ni]] = v[mi][ni] + acc[mi][ni][q];
    }
  } else {
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int off = rowtab[wm0 + mi * 32 + acc_row(q, lane)];  // one row per half-wave and (mi, q)
        if (off < 0) continue;
        float v[TN];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) v[ni] = mine[off + col_off[ni]];
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
          if (col_ok[ni]) mine[off + col_off[ni]] = v[ni] + acc[mi][ni][q];
      }
  }
  __syncthreads();
  float* out = a.partial + (((int64_t)n * a.tiles_i + it) * a.tiles_j + jt) * a.rsz;
  const int used = g.nch * plane;
  for (int e = tid; e < used; e += kThreads) {
    float v = reg0[e];
#pragma unroll
    for (int k = 1; k < kCopies; ++k) v += reg0[k * a.rsz + e];
    out[e] = v;
  }
}

// p / d for 0 <= p < 2^23 and 0 < d: a float reciprocal and one correction step instead of an integer division
__device__ __forceinline__ int div_small(int p, int d, float inv_d) {
  int q = (int)((float)p * inv_d);
  const int r = p - q * d;
  q += (r >= d) - (r < 0);
  return q;
}

// dx[n][c][h][w] = sum of the region entries that stand for that pixel, over the tiles covering it, in ascending
// (row tile, column tile) order.  (What fold_region computes, with the per-tile divisions reduced to a few.)
template <typename T>
__global__ __launch_bounds__(kThreads) void fold_gather_kernel(FoldArgs a, float inv_ow) {
  const int64_t total = (int64_t)a.n * a.c * a.h * a.wd;
  const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (e >= total) return;
  const int w = (int)(e % a.wd);
  int64_t t = e / a.wd;
  const int h = (int)(t % a.h);
  t /= a.h;
  const int c = (int)(t % a.c);
  const int n = (int)(t / a.c);
  const int RS = a.r * a.s;
  const int it_lo = (c * RS) / kFoldBM, it_hi = ((c + 1) * RS - 1) / kFoldBM;
  float acc = 0.f;
  for (int it = it_lo; it <= it_hi; ++it) {
    // the row tile's channels and, if it holds a single channel, its kernel rows
    const int i_first = it * kFoldBM, i_last = min(i_first + kFoldBM, a.K) - 1;
    const int c_lo = i_first / RS, nch = i_last / RS - c_lo + 1;
    int r_lo = 0, r_hi = a.r - 1;
    if (nch == 1) r_lo = (i_first - c_lo * RS) / a.s, r_hi = (i_last - c_lo * RS) / a.s;
    // output rows oh = h + pad_h - r that reach input row h through those kernel rows
    const int oh_min = max(h + a.ph - r_hi, 0), oh_max = min(h + a.ph - r_lo, a.oh - 1);
    if (oh_min > oh_max) continue;
    const int jt_lo = (oh_min * a.ow) / kFoldBN, jt_hi = (oh_max * a.ow + a.ow - 1) / kFoldBN;
    const float* src = a.partial + (((int64_t)n * a.tiles_i + it) * a.tiles_j + jt_lo) * a.rsz;
    for (int jt = jt_lo; jt <= jt_hi; ++jt, src += a.rsz) {
      const int oh_first = div_small(jt * kFoldBN, a.ow, inv_ow);
      const int oh_last = div_small(min(jt * kFoldBN + kFoldBN, a.P) - 1, a.ow, inv_ow);
      const int nrows = (oh_last - oh_first) + (r_hi - r_lo) + 1;
      const int row = h - (oh_first + r_lo - a.ph);
      if (row < 0 || row >= nrows) continue;
      acc += src[((c - c_lo) * nrows + row) * a.wreg + (w + a.pw)];
    }
  }
  if (a.dact) acc = act_grad(a.dact, ld(static_cast<const T*>(a.dact_ref) + e), acc);
  st(static_cast<T*>(a.dx) + e, acc);
}

bool bwd_data_fold_plan(const ConvGeom& g, FoldPlan* p) {
  if (g.M < 32) return false;  // short contractions leave the fold, not the product, as the bulk of the work
  if (g.P >= (1 << 23)) return false;  // pixel indices stay exact in float (div_small)
  const int RS = g.r * g.s;
  const int tiles_i = (int)ceil_div(g.K, kFoldBM), tiles_j = (int)ceil_div(g.P, kFoldBN);
  // largest region over all tiles: (channels x kernel rows) of a row tile, plus the output rows a column tile spans
  const int wreg = g.ow + g.s - 1;
  int span = 0;
  for (int jt = 0; jt < tiles_j; ++jt) {
    const FoldRegion f = fold_region(0, jt, (int)g.K, (int)g.P, RS, g.s, g.r, g.ow, g.ph);
    span = std::max(span, f.nrows - (f.r_hi - f.r_lo + 1));  // last output row - first output row of the tile
  }
  int64_t rows = 0;
  for (int it = 0; it < tiles_i; ++it) {
    const FoldRegion f = fold_region(it, 0, (int)g.K, (int)g.P, RS, g.s, g.r, g.ow, g.ph);
    rows = std::max<int64_t>(rows, (int64_t)f.nch * (span + f.r_hi - f.r_lo + 1));
  }
  if (rows * wreg > (1 << 20)) return false;
  const int rsz = (int)(rows * wreg);
  if ((size_t)rsz * kCopies * sizeof(float) > 60 * 1024) return false;
  // the regions must stay a small fraction of the patch-matrix gradient they replace
  if ((int64_t)rsz * 4 > (int64_t)kFoldBM * kFoldBN) return false;
  p->tiles_i = tiles_i, p->tiles_j = tiles_j, p->rsz = rsz, p->wreg = wreg;
  p->partial_bytes = (size_t)g.n * tiles_i * tiles_j * rsz * sizeof(float);
  const size_t slabs = 2 * (size_t)(LdsTile<kFoldBM, kFoldBK, false>::SIZE + LdsTile<kFoldBN, kFoldBK, false>::SIZE) * sizeof(float);
  p->lds_bytes = std::max(slabs, (size_t)rsz * kCopies * sizeof(float) + kFoldBM * sizeof(int));
  return (int64_t)g.n * tiles_i * tiles_j <= 0x7fffffffLL;
}

vcnn_status launch_bwd_data_fold(const FoldPlan& p, int dtype, const ConvGeom& g, const void* w, const void* dy, void* dx,
                                 float* partial, hipStream_t st, int dact, const void* dact_ref) {
  FoldArgs a{};
  a.w = w, a.dy = dy, a.partial = partial, a.dx = dx;
  a.dact = dact_ref ? dact : 0, a.dact_ref = dact_ref;
  a.n = g.n, a.c = g.c, a.h = g.h, a.wd = g.w, a.m = (int)g.M, a.r = g.r, a.s = g.s, a.ph = g.ph, a.pw = g.pw;
  a.oh = g.oh, a.ow = g.ow, a.P = (int)g.P, a.K = (int)g.K;
  a.tiles_i = p.tiles_i, a.tiles_j = p.tiles_j, a.rsz = p.rsz, a.wreg = p.wreg;
  const dim3 grid((unsigned)((int64_t)g.n * p.tiles_i * p.tiles_j)), block(kThreads);
  const bool bf = dtype == VCNN_BF16;
  const bool vec = bf ? g.K % 4 == 0 && group_aligned<bf16>(w) : g.K >= 4 && (reinterpret_cast<uintptr_t>(w) & 3) == 0;
  // Rows i and i + 32 of one channel are taps (r1, s1), (r2, s2) with (r2 - r1) * s + (s2 - s1) = 32; their entries
  // for pixels p, p' land on one input pixel iff p' - p = (r2 - r1) * ow + (s2 - s1).  A wave's pixels span 64
  // consecutive ones, so beyond that distance the two rows' adds of one step cannot meet.
  bool mi_indep = true;
  for (int dr = 32 / g.s; dr <= 32 / g.s + 1; ++dr) {
    const int ds = 32 - dr * g.s;
    if (ds > -g.s && ds < g.s && dr < g.r && std::abs(dr * g.ow + ds) < 64) mi_indep = false;
  }
  auto go = [&](auto kernel) {
    if (p.lds_bytes > 48 * 1024)  // opt in to more than the default dynamic LDS limit (idempotent, host-side only)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
    hipLaunchKernelGGL(kernel, grid, block, p.lds_bytes, st, a);
  };
  const bool bvec = !bf && g.P >= 4 && (reinterpret_cast<uintptr_t>(dy) & 3) == 0;
  if (bf) {
    if (vec && mi_indep) go(bwd_data_fold_kernel<true, false, true, bf16>);
    else if (vec) go(bwd_data_fold_kernel<true, false, false, bf16>);
    else go(bwd_data_fold_kernel<false, false, false, bf16>);
  } else if (bvec) {
    if (vec && mi_indep) go(bwd_data_fold_kernel<true, true, true, float>);
    else if (vec) go(bwd_data_fold_kernel<true, true, false, float>);
    else go(bwd_data_fold_kernel<false, true, false, float>);
  } else {
    if (vec && mi_indep) go(bwd_data_fold_kernel<true, false, true, float>);
    else if (vec) go(bwd_data_fold_kernel<true, false, false, float>);
    else go(bwd_data_fold_kernel<false, false, false, float>);
  }
  if (vcnn_status s = check_launch("bwd_data_fold")) return s;
  const int64_t total = (int64_t)g.n * g.c * g.h * g.w;
  const dim3 grid2((unsigned)ceil_div(total, kThreads));
  const float inv_ow = 1.0f / (float)g.ow;
  if (bf) hipLaunchKernelGGL(fold_gather_kernel<bf16>, grid2, block, 0, st, a, inv_ow);
  else hipLaunchKernelGGL(fold_gather_kernel<float>, grid2, block, 0, st, a, inv_ow);
  return check_launch("fold_gather");
}

}  // namespace vcnn
