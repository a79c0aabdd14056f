// Dense matrix products of the vectorized layer on the CDNA4 matrix cores (fp32 in, fp32 accumulate).
//
//   forward   (Eq. 2 / Eq. 4):  Y[M x N]    = W[M x K] * col[K x N]  (+ bias, sigma), stored as [N][M][P]
//   bwd data  (phi_c^{-1} arg): dcol[K x N] = W^T * dY
//   bwd filter:                 dW[M x K]   = dY * col^T  (contraction over the N = batch*OH*OW axis)
//   fully connected layers: the same products with plain row-major operands.
//
// All of them run v_mfma_f32_32x32x2_f32 on LDS-staged, double-buffered slabs (see mma_core.h): the
// global loads of slab t+1 are issued before the MFMAs of slab t and written to the other LDS buffer
// afterwards, so a block synchronises once per slab.

#include <type_traits>

#include "common.h"
#include "elem.h"
#include "mma_core.h"

namespace vcnn {

static constexpr int kThreads = 256;

__device__ __forceinline__ int64_t jmap(int j, int P, int64_t s_img, int64_t s_j) {
  if (P > 0) {
    const int q = j / P;
    return (int64_t)q * s_img + (int64_t)(j - q * P) * s_j;
  }
  return (int64_t)j * s_j;
}

// Consecutive block ids are dealt round-robin to the 8 XCDs (each with its own L2).  Remap so that a
// run of consecutive tile ids - which share operand panels - stays on one XCD.
__device__ __forceinline__ int xcd_remap(int bid, int total) {
  constexpr int X = 8;
  const int per = total / X;           // tiles per XCD in the evenly divisible part
  const int body = per * X;
  if (bid >= body) return bid;         // ragged tail keeps its id
  return (bid % X) * per + bid / X;
}

// TI: element type of A and B in memory (float or bf16); TO: element type of C.  All arithmetic is fp32.
template <int BM, int BN, int BK, int WM, int WN, bool A_KC, bool B_KC, bool A_VEC, bool B_VEC, typename TI, typename TO>
__global__ __launch_bounds__(kThreads, BK == 16 ? 4 : 1) void gemm_f32_kernel(GemmArgs a, int tiles_m, int tiles_total) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  using LA = LdsTile<BM, BK, A_KC>;
  using LB = LdsTile<BN, BK, B_KC>;
  using SA = Stager<BM, BK, kThreads, A_KC, A_VEC>;
  using SB = Stager<BN, BK, kThreads, B_KC, B_VEC>;
  constexpr int TM = WM / 32, TN = WN / 32;
  extern __shared__ float4 smem4[];
  float* smem = reinterpret_cast<float*>(smem4);
  // Buffers are addressed as smem + offset (not through a pointer table) so that the compiler keeps
  // them in the LDS address space and emits ds_read/ds_write rather than flat accesses.
  float* const As0 = smem;
  float* const Bs0 = smem + 2 * LA::SIZE;

  const TI* gA = static_cast<const TI*>(a.A);
  const TI* gB = static_cast<const TI*>(a.B);
  TO* gC = static_cast<TO*>(a.C);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tile = xcd_remap(blockIdx.x, tiles_total);
  const int i0 = (tile % tiles_m) * BM;
  const int j0 = (tile / tiles_m) * BN;
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;

  SA sa;
  SB sb;
  sa.init(tid);
  sb.init(tid);
  // Element offsets of every slot at k = 0.  Slots whose row lies outside the matrix point at row 0 and
  // are zeroed when the slab is written to LDS, so the loads themselves are unconditional and
  // branch-free (they stay in flight across the MFMAs of the current slab).
  int64_t a_off[SA::SLOTS], b_off[SB::SLOTS];
  bool a_row_ok[SA::SLOTS], b_row_ok[SB::SLOTS];
#pragma unroll
  for (int e = 0; e < SA::SLOTS; ++e) {
    const int i = i0 + sa.row_of(e, 0);
    a_row_ok[e] = i < a.M;
    a_off[e] = (int64_t)(a_row_ok[e] ? i : 0) * a.a_si;
  }
#pragma unroll
  for (int e = 0; e < SB::SLOTS; ++e) {
    const int j = j0 + sb.row_of(e, 0);
    b_row_ok[e] = j < a.N;
    b_off[e] = jmap(b_row_ok[e] ? j : 0, a.b_P, a.b_simg, a.b_sj);
  }
  // B contiguous along j and fetched four columns at a time (B_VEC, !B_KC; float: at any dword boundary): every slot
  // of a thread holds the same four columns j .. j+3.  If they run over the end of the matrix or of a sample (per-sample
  // [k][P] maps with P not a multiple of 4) they are fetched one by one from their own offsets.
  bool b_whole = true;
  int64_t b_off1[4] = {0, 0, 0, 0};
  bool b_ok1[4] = {false, false, false, false};
  if constexpr (B_VEC && !B_KC && std::is_same<TI, float>::value) {
    const int j = j0 + sb.c;
    b_whole = j + 3 < a.N && (a.b_P == 0 || j % a.b_P + 3 < a.b_P);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      b_ok1[u] = j + u < a.N;
      b_off1[u] = jmap(b_ok1[u] ? j + u : 0, a.b_P, a.b_simg, a.b_sj);
    }
  }

  auto fetch = [&](int k0) {
#pragma unroll
    for (int e = 0; e < SA::SLOTS; ++e) {
      const int k = k0 + sa.k_of(e, 0);
      sa.ok[e] = a_row_ok[e] && k < a.K;
      const TI* src = gA + a_off[e] + (int64_t)min(k, (A_VEC && A_KC) ? a.K - 4 : a.K - 1) * a.a_sk;
      if (A_VEC) {
        const float4 t = ld4(src);
        sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
      } else {
        sa.v[e][0] = ld(src);
      }
    }
#pragma unroll
    for (int e = 0; e < SB::SLOTS; ++e) {
      const int k = k0 + sb.k_of(e, 0);
      sb.ok[e] = b_row_ok[e] && k < a.K;
      const TI* src = gB + b_off[e] + (int64_t)min(k, (B_VEC && B_KC) ? a.K - 4 : a.K - 1) * a.b_sk;
      if constexpr (B_VEC && !B_KC && std::is_same<TI, float>::value) {
        if (b_whole) {
          const float4 t = ld4_dword_aligned(src);
          sb.v[e][0] = t.x, sb.v[e][1] = t.y, sb.v[e][2] = t.z, sb.v[e][3] = t.w;
        } else {
          const int64_t ko = (int64_t)min(k, a.K - 1) * a.b_sk;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const float t = ld(gB + b_off1[u] + ko);
            sb.v[e][u] = b_ok1[u] ? t : 0.f;
          }
        }
      } else if constexpr (B_VEC) {
        const float4 t = ld4(src);
        sb.v[e][0] = t.x, sb.v[e][1] = t.y, sb.v[e][2] = t.z, sb.v[e][3] = t.w;
      } else {
        sb.v[e][0] = ld(src);
      }
    }
  };

  f32x16 acc[TM][TN];
  zero_acc<TM, TN>(acc);

  const int ktiles = (a.K + BK - 1) / BK;
  fetch(0);
  sa.store(As0);
  sb.store(Bs0);
  __syncthreads();
  for (int kt = 0; kt < ktiles; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < ktiles) fetch((kt + 1) * BK);
    mma_slab<BM, BN, BK, TM, TN, A_KC, B_KC>(As0 + cur * LA::SIZE, Bs0 + cur * LB::SIZE, wm0, wn0, lane, acc);
    if (kt + 1 < ktiles) {
      sa.store(As0 + (cur ^ 1) * LA::SIZE);
      sb.store(Bs0 + (cur ^ 1) * LB::SIZE);
    }
    __syncthreads();
  }

  const int l32 = lane & 31;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int j = j0 + wn0 + ni * 32 + l32;
    if (j >= a.N) continue;
    const int64_t cj = jmap(j, a.c_P, a.c_simg, a.c_sj);
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int i = i0 + wm0 + mi * 32 + acc_row(q, lane);
        if (i < a.M) {
          float v = acc[mi][ni][q];
          if (a.bias) v += a.bias[i];
          if (a.relu) v = fmaxf(v, 0.f);
          const int64_t at = (int64_t)i * a.c_si + cj;
          if (a.dact) v = act_grad(a.dact, ld(static_cast<const TO*>(a.dact_ref) + at), v);
          st(gC + at, v);
        }
      }
  }
}

template <int BM, int BN, int BK, bool A_KC, bool B_KC>
static constexpr size_t gemm_lds_bytes() {
  return 2 * (size_t)(LdsTile<BM, BK, A_KC>::SIZE + LdsTile<BN, BK, B_KC>::SIZE) * sizeof(float);
}

// Opts a kernel in to more than the default dynamic LDS limit, once per kernel.
template <typename K>
static void allow_lds(K kernel, size_t bytes, bool& done) {
  if (bytes > 48 * 1024 && !done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)bytes);
    done = true;
  }
}

template <int BM, int BN, int BK, int WM, int WN, bool A_KC, bool B_KC, bool A_VEC, bool B_VEC, typename TI, typename TO>
static void launch_one(const GemmArgs& a, hipStream_t st) {
  const int tiles_m = (int)ceil_div(a.M, BM);
  const int64_t blocks = (int64_t)tiles_m * ceil_div(a.N, BN);
  const size_t lds = gemm_lds_bytes<BM, BN, BK, A_KC, B_KC>();
  auto kernel = gemm_f32_kernel<BM, BN, BK, WM, WN, A_KC, B_KC, A_VEC, B_VEC, TI, TO>;
  static bool opted_in = false;  // one flag per instantiation of this launcher, i.e. per kernel
  allow_lds(kernel, lds, opted_in);
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kThreads), lds, st, a, tiles_m, (int)blocks);
}

template <int BM, int BN, int BK, int WM, int WN, bool A_KC, bool B_KC, bool A_VEC, bool B_VEC>
static void launch_typed(const GemmArgs& a, hipStream_t st) {
  if (a.in_dtype == VCNN_BF16) {
    if (a.out_dtype == VCNN_BF16)
      launch_one<BM, BN, BK, WM, WN, A_KC, B_KC, A_VEC, B_VEC, bf16, bf16>(a, st);
    else
      launch_one<BM, BN, BK, WM, WN, A_KC, B_KC, A_VEC, B_VEC, bf16, float>(a, st);
  } else {
    launch_one<BM, BN, BK, WM, WN, A_KC, B_KC, A_VEC, B_VEC, float, float>(a, st);
  }
}

template <int BM, int BN, int BK, int WM, int WN, bool A_KC, bool B_KC>
static void launch_vec(const GemmArgs& a, bool av, bool bv, hipStream_t st) {
  if (av && bv)
    launch_typed<BM, BN, BK, WM, WN, A_KC, B_KC, true, true>(a, st);
  else if (av)
    launch_typed<BM, BN, BK, WM, WN, A_KC, B_KC, true, false>(a, st);
  else if (bv)
    launch_typed<BM, BN, BK, WM, WN, A_KC, B_KC, false, true>(a, st);
  else
    launch_typed<BM, BN, BK, WM, WN, A_KC, B_KC, false, false>(a, st);
}

template <int BM, int BN, int BK, int WM, int WN>
static void launch_cfg(const GemmArgs& a, bool a_kc, bool b_kc, bool av, bool bv, hipStream_t st) {
  if (a_kc && b_kc)
    launch_vec<BM, BN, BK, WM, WN, true, true>(a, av, bv, st);
  else if (a_kc)
    launch_vec<BM, BN, BK, WM, WN, true, false>(a, av, bv, st);
  else if (b_kc)
    launch_vec<BM, BN, BK, WM, WN, false, true>(a, av, bv, st);
  else
    launch_vec<BM, BN, BK, WM, WN, false, false>(a, av, bv, st);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
// -------------------------------------------------------------------------------------------------
// Small products (the fully connected layers at the experiments' batch sizes: a few MFLOP).  Their cost
// is latency, not arithmetic: few tiles, and in the slab kernel above a chain of load -> barrier ->
// MFMA rounds as long as the contraction.  Here a block owns one 32 x 32 (or 16 x 16) tile of C and its waves
// (4 to 8, more for longer contractions) split the contraction between them; every wave reads its operand
// fragments straight from global memory, several groups of 8 contraction steps in flight at once (no LDS
// staging, no barrier in the loop), and the partial tiles are added in wave order through LDS.
// -------------------------------------------------------------------------------------------------
// GemmArgs::row_sums: B gets a virtual column j = N of ones, whose products - the row sums of A - go to
// row_sums[i] (a fully connected layer's bias gradient comes out of its weight-gradient product this way).
// T16: 16 x 16 tiles on v_mfma_f32_16x16x4_f32 instead of 32 x 32 on v_mfma_f32_32x32x2_f32, for products with so
// few 32 x 32 tiles that most compute units would stay idle (four times the blocks, a quarter of the rows each).
typedef float f32x4s __attribute__((ext_vector_type(4)));
template <bool T16, bool A_KC, bool B_KC, bool A_VEC, bool B_VEC, typename TI, typename TO>
__device__ __forceinline__ void small_tile(const GemmArgs& a, int tile, int tiles_m, int kper, float* red) {
  constexpr int TS = T16 ? 16 : 32;    // tile side
  constexpr int KL = T16 ? 4 : 2;      // lanes that share a row (each takes every KL-th group of four indices)
  constexpr int GK = 4 * KL;           // contraction indices per group = 4 MFMA steps
  constexpr int NQ = T16 ? 4 : 16;     // accumulator registers per lane
  const int waves = blockDim.x >> 6;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & (TS - 1), kq = lane / TS;
  const int i0 = (tile % tiles_m) * TS, j0 = (tile / tiles_m) * TS;
  const int i = i0 + lr, j = j0 + lr;  // this lane's row of A and column of B
  const bool i_ok = i < a.M, j_ok = j < a.N;
  const bool j_ones = a.row_sums != nullptr && j == a.N;
  const TI* A = static_cast<const TI*>(a.A) + (int64_t)(i_ok ? i : 0) * a.a_si;
  const TI* B = static_cast<const TI*>(a.B) + (int64_t)(j_ok ? j : 0) * a.b_sj;
  const int ks = wave * kper, ke = min(a.K, ks + kper);  // kper is a multiple of GK

  typename std::conditional<T16, f32x4s, f32x16>::type acc;
#pragma unroll
  for (int q = 0; q < NQ; ++q) acc[q] = 0.f;

  // one group = GK contraction indices = 4 MFMA steps; the lanes of a row feed k0 + 4 * kq + step
  auto load4 = [&](const TI* base, int64_t sk, bool kc, bool vec, bool row_ok, bool ones, int k0, float (&v)[4]) {
    const int kb = k0 + 4 * kq;
    if (kc && vec) {
      const bool ok = row_ok && kb < ke;  // K and the split are multiples of 4: a group of four is in or out as a whole
      const float4 t = ld4(base + (ok ? kb : 0));
      v[0] = ok ? t.x : 0.f, v[1] = ok ? t.y : 0.f, v[2] = ok ? t.z : 0.f, v[3] = ok ? t.w : 0.f;
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool ok = row_ok && kb + u < ke;
        const float t = ld(base + (ok ? (int64_t)(kb + u) * sk : 0));
        v[u] = ok ? t : 0.f;
      }
    }
    if (ones) {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = kb + u < ke ? 1.f : 0.f;
    }
  };
  constexpr int U = 8;  // groups in flight
  for (int k0 = ks; k0 < ke; k0 += GK * U) {
    float av[U][4], bv[U][4];
    const int ng = min(U, (ke - k0 + GK - 1) / GK);  // groups with work (wave-uniform): short shares skip the rest
#pragma unroll
    for (int g = 0; g < U; ++g)
      if (g < ng) {
        load4(A, a.a_sk, A_KC, A_VEC, i_ok, false, k0 + GK * g, av[g]);
        load4(B, a.b_sk, B_KC, B_VEC, j_ok, j_ones, k0 + GK * g, bv[g]);
      }
#pragma unroll
    for (int g = 0; g < U; ++g)
      if (g < ng) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if constexpr (T16) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[g][u], bv[g][u], acc, 0, 0, 0);
          else acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g][u], bv[g][u], acc, 0, 0, 0);
        }
      }
  }

  if (wave > 0) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) red[((wave - 1) * NQ + q) * 64 + lane] = acc[q];
  }
  __syncthreads();
  if (wave > 0) return;
  for (int w = 0; w < waves - 1; ++w)
#pragma unroll
    for (int q = 0; q < NQ; ++q) acc[q] += red[(w * NQ + q) * 64 + lane];
  if (!j_ok && !j_ones) return;
  TO* C = static_cast<TO*>(a.C);
  // what the epilogue reads (bias, the activation below) is requested for all rows at once, at clamped addresses,
  // before any of it is used: one memory latency instead of one per accumulator register
  float bq[NQ], rq[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) bq[q] = 0.f, rq[q] = 0.f;
  if (a.bias) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) bq[q] = a.bias[min(i0 + (T16 ? 4 * kq + q : acc_row(q, lane)), a.M - 1)];
  }
  if (a.dact && !j_ones) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int row = min(i0 + (T16 ? 4 * kq + q : acc_row(q, lane)), a.M - 1);
      rq[q] = ld(static_cast<const TO*>(a.dact_ref) + (int64_t)row * a.c_si + (int64_t)j * a.c_sj);
    }
  }
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int row = i0 + (T16 ? 4 * kq + q : acc_row(q, lane));
    if (row < a.M) {
      float v = acc[q];
      if (j_ones) {
        a.row_sums[row] = v;
        continue;
      }
      v += bq[q];
      if (a.relu) v = fmaxf(v, 0.f);
      const int64_t at = (int64_t)row * a.c_si + (int64_t)j * a.c_sj;
      if (a.dact) v = act_grad(a.dact, rq[q], v);
      st(C + at, v);
    }
  }
}

template <bool A_KC, bool B_KC, bool A_VEC, bool B_VEC, typename TI, typename TO>
__global__ __launch_bounds__(1024) void gemm_small_kernel(GemmArgs a, int tiles_m, int kper, int t16) {
  extern __shared__ float red[];  // [waves - 1][16][64]
  if (t16) small_tile<true, A_KC, B_KC, A_VEC, B_VEC, TI, TO>(a, blockIdx.x, tiles_m, kper, red);
  else small_tile<false, A_KC, B_KC, A_VEC, B_VEC, TI, TO>(a, blockIdx.x, tiles_m, kper, red);
}

// Both products of a fully connected layer's backward pass in one launch: tiles_w blocks compute the weight
// gradient dW = dY^T X (with the bias gradient as its column of ones), tiles_x blocks the input gradient
// dX = dY W.  The two are independent, and at these sizes neither fills the chip alone.  The product with the
// longer contraction takes the low block ids: when the grid is a little larger than what is resident at once,
// the blocks that start late are then the short ones.
template <bool A_VEC, typename TI>
__global__ __launch_bounds__(1024) void fc_bwd_small_kernel(GemmArgs gw, GemmArgs gx, int tiles_w, int tiles_m_w,
                                                            int kper_w, int tiles_x, int tiles_m_x, int kper_x,
                                                            int x_first, int w16, int x16) {
  extern __shared__ float red[];
  const int b = blockIdx.x;
  const bool is_w = x_first ? b >= tiles_x : b < tiles_w;
  if (is_w) {
    const int t = x_first ? b - tiles_x : b;
    if (w16) small_tile<true, false, false, false, false, TI, float>(gw, t, tiles_m_w, kper_w, red);
    else small_tile<false, false, false, false, false, TI, float>(gw, t, tiles_m_w, kper_w, red);
  } else {
    const int t = x_first ? b : b - tiles_w;
    if (x16) small_tile<true, true, false, A_VEC, false, TI, TI>(gx, t, tiles_m_x, kper_x, red);
    else small_tile<false, true, false, A_VEC, false, TI, TI>(gx, t, tiles_m_x, kper_x, red);
  }
}

// 4 to 8 waves split the contraction, 8 from 128 indices on (16 measured no faster and need 61 KB of LDS for the
// partial tiles)
static int small_waves(int K) { return (int)std::min<int64_t>(8, std::max<int64_t>(4, ceil_div(K, 16))); }
static int64_t small_tiles(const GemmArgs& a) { return ceil_div(a.M, 32) * ceil_div(a.N + (a.row_sums ? 1 : 0), 32); }
// At most 64 tiles of 32 x 32 leave three quarters of the chip idle: 16 x 16 tiles then.  The choice depends on the
// product alone, so a product returns the same bits whichever launch carries it.
static bool small_use16(const GemmArgs& a) { return small_tiles(a) <= 64; }
static int small_side(const GemmArgs& a) { return small_use16(a) ? 16 : 32; }
static int64_t small_blocks(const GemmArgs& a) {
  const int ts = small_side(a);
  return ceil_div(a.M, ts) * ceil_div(a.N + (a.row_sums ? 1 : 0), ts);
}
// a wave's share of the contraction: a multiple of the indices one group of four MFMA steps covers (8 or 16)
static int small_kper(const GemmArgs& a, int waves) {
  const int gk = small_use16(a) ? 16 : 8;
  return (int)ceil_div(ceil_div(a.K, waves), gk) * gk;
}

template <bool A_KC, bool B_KC, bool A_VEC, bool B_VEC>
static void launch_small_t(const GemmArgs& a, hipStream_t st) {
  const int tiles_m = (int)ceil_div(a.M, small_side(a));
  const int64_t tiles = small_blocks(a);
  const int waves = small_waves(a.K);
  const int kper = small_kper(a, waves);
  const int t16 = small_use16(a);
  const dim3 grid((unsigned)tiles), block(64 * waves);
  const size_t lds = (size_t)(waves - 1) * 16 * 64 * sizeof(float);
  const bool in16 = a.in_dtype == VCNN_BF16, out16 = a.out_dtype == VCNN_BF16;
  if (in16 && out16)
    hipLaunchKernelGGL((gemm_small_kernel<A_KC, B_KC, A_VEC, B_VEC, bf16, bf16>), grid, block, lds, st, a, tiles_m, kper, t16);
  else if (in16)
    hipLaunchKernelGGL((gemm_small_kernel<A_KC, B_KC, A_VEC, B_VEC, bf16, float>), grid, block, lds, st, a, tiles_m, kper, t16);
  else
    hipLaunchKernelGGL((gemm_small_kernel<A_KC, B_KC, A_VEC, B_VEC, float, float>), grid, block, lds, st, a, tiles_m, kper, t16);
}

static void launch_small(const GemmArgs& a, bool a_kc, bool b_kc, bool av, bool bv, hipStream_t st) {
  // 16-byte loads only matter (and are only defined here) for contraction-contiguous operands
  av = av && a_kc, bv = bv && b_kc;
  if (a_kc && b_kc) {
    if (av && bv) launch_small_t<true, true, true, true>(a, st);
    else launch_small_t<true, true, false, false>(a, st);
  } else if (a_kc) {
    if (av) launch_small_t<true, false, true, false>(a, st);
    else launch_small_t<true, false, false, false>(a, st);
  } else if (b_kc) {
    if (bv) launch_small_t<false, true, false, true>(a, st);
    else launch_small_t<false, true, false, false>(a, st);
  } else {
    launch_small_t<false, false, false, false>(a, st);
  }
}

bool gemm_is_small(const GemmArgs& a) {
  return a.b_P == 0 && a.c_P == 0 && small_tiles(a) <= 512 && (int64_t)a.M * a.N * a.K <= (int64_t)1 << 27;
}

static bool in_aligned(const void* p, int dtype) { return dtype == VCNN_BF16 ? group_aligned<bf16>(p) : group_aligned<float>(p); }

vcnn_status launch_gemm_f32(const GemmArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(VCNN_ERR_SHAPE, "gemm: empty operand");
  const bool a_kc = (a.a_sk == 1) && (a.a_si != 1);
  const bool b_kc = (a.b_sk == 1) && (a.b_sj != 1);
  // 16-byte loads need the contiguous axis to come in aligned groups of four that never straddle a
  // row (or, for the [N][M][P] maps, a sample) boundary.
  bool av, bv;
  if (a_kc)
    av = in_aligned(a.A, a.in_dtype) && a.a_si % 4 == 0 && a.K % 4 == 0;
  else
    av = in_aligned(a.A, a.in_dtype) && a.a_si == 1 && a.a_sk % 4 == 0 && a.M % 4 == 0;
  if (b_kc)
    bv = in_aligned(a.B, a.in_dtype) && a.b_P == 0 && a.b_sj % 4 == 0 && a.K % 4 == 0;
  else if (a.in_dtype == VCNN_F32)  // 16-byte loads at any dword boundary; groups that straddle are split in the kernel
    bv = (reinterpret_cast<uintptr_t>(a.B) & 3) == 0 && a.b_sj == 1 && a.N >= 4;
  else
    bv = in_aligned(a.B, a.in_dtype) && a.b_sj == 1 && a.b_sk % 4 == 0 && a.N % 4 == 0 &&
         (a.b_P == 0 || (a.b_P % 4 == 0 && a.b_simg % 4 == 0));
  // Small products (the fully connected layers at batch 128) would fill only a handful of large
  // tiles; 64x64 tiles spread them over more compute units.
  const int64_t big_tiles = ceil_div(a.M, 128) * ceil_div(a.N, 128);
  if (gemm_is_small(a)) {
    launch_small(a, a_kc, b_kc, av, bv, st);
    return check_launch("gemm_small");
  }
  if (a.row_sums) return fail(VCNN_ERR_UNSUPPORTED, "gemm: row sums are only built into the small-product kernel");
  if (a.M > 32 && a.N <= 4096 && big_tiles < 128)
    launch_cfg<64, 64, 32, 32, 32>(a, a_kc, b_kc, av, bv, st);
  else if (a.M <= 32)
    launch_cfg<32, 256, 32, 32, 64>(a, a_kc, b_kc, av, bv, st);
  else if (a.M <= 64 && ceil_div(a.N, 256) < 256)  // too few 256-wide tiles to occupy the compute units: halve them
    launch_cfg<64, 128, 32, 32, 64>(a, a_kc, b_kc, av, bv, st);
  else if (a.M <= 64)
    launch_cfg<64, 256, 32, 64, 64>(a, a_kc, b_kc, av, bv, st);
  else
    launch_cfg<128, 128, 16, 64, 64>(a, a_kc, b_kc, av, bv, st);
  return check_launch("gemm_f32");
}

// -------------------------------------------------------------------------------------------------
// Filter gradient: dW[m][k] = sum_j dY(m, j) * col[k][j].  Both operands are contiguous along the
// contraction index j; dY lives in [N][M][P] layout, so j = n*P + p addresses dy[(n*M + m)*P + p].
// blockIdx.y selects a range of columns; each range writes its own partial product and a second
// kernel adds the partials in ascending order, which keeps the result independent of scheduling.
// -------------------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WM, int WN, bool VEC, typename T>
__global__ __launch_bounds__(kThreads) void bwd_filter_f32_kernel(ConvGeom g, const T* __restrict__ dy,
                                                                  const T* __restrict__ col, const T* __restrict__ xin,
                                                                  float* __restrict__ out, int tiles_m, int chunk) {
  static_assert((BM / WM) * (BN / WN) * 64 == kThreads, "four waves per block");
  using LA = LdsTile<BM, BK, true>;
  using LB = LdsTile<BN, BK, true>;
  using SA = Stager<BM, BK, kThreads, true, VEC>;
  using SB = Stager<BN, BK, kThreads, true, VEC>;
  constexpr int TM = WM / 32, TN = WN / 32;
  extern __shared__ float4 smem4[];
  float* smem = reinterpret_cast<float*>(smem4);
  // Buffers are addressed as smem + offset (not through a pointer table) so that the compiler keeps
  // them in the LDS address space and emits ds_read/ds_write rather than flat accesses.
  float* const As0 = smem;
  float* const Bs0 = smem + 2 * LA::SIZE;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int i0 = tm * BM, k0 = tn * BN;  // i: output map (row of dW); k: patch-matrix row (column of dW)
  const int wm0 = (wave % (BM / WM)) * WM;
  const int wn0 = (wave / (BM / WM)) * WN;
  const int64_t js = (int64_t)blockIdx.y * chunk;
  const int64_t je = min((int64_t)g.N, js + chunk);
  const int M = (int)g.M, K = (int)g.K;
  const int P = (int)g.P;

  SA sa;
  SB sb;
  sa.init(tid);
  sb.init(tid);
  // (n, p) of this thread's first contraction index (sa.c == sb.c: same position inside the slab).
  int64_t j = js + sa.c;
  int n = (int)(j / P);
  int p = (int)(j - (int64_t)n * P);

  // B operand: the patch matrix col[k][j], or - for an unpadded 1 x 1 layer, whose patch matrix is the input itself
  // sample by sample - x[(n*K + k)*P + p] read in place (xin != nullptr).
  auto b_src = [&](int k, int nn, int pp, int64_t jj) {
    return xin ? xin + ((int64_t)nn * K + k) * P + pp : col + (int64_t)k * g.N + jj;
  };
  auto fetch = [&]() {
    // Out-of-range slots load from a clamped, valid address and are zeroed when written to LDS.  VEC: a group of
    // four consecutive contraction indices is one 16-byte load when it lies inside one sample and inside the range
    // (float: at any dword boundary; bf16: P and the range are multiples of 4, so groups never straddle); a group
    // that runs over the end of a sample or of the range is fetched element by element.
    const bool jin = j < je;
    const int nn = jin ? n : 0, pp = jin ? p : 0;
    const int64_t jj = jin ? j : 0;
    const bool whole = !VEC || (j + 3 < je && p + 3 < P);
    if (whole || !jin) {
#pragma unroll
      for (int e = 0; e < SA::SLOTS; ++e) {
        const int m = i0 + sa.line(e);
        sa.ok[e] = jin && m < M;
        const T* src = dy + ((int64_t)nn * M + min(m, M - 1)) * P + pp;
        if constexpr (VEC) {
          float4 t;
          if constexpr (std::is_same<T, float>::value) t = ld4_dword_aligned(src);
          else t = ld4(src);
          sa.v[e][0] = t.x, sa.v[e][1] = t.y, sa.v[e][2] = t.z, sa.v[e][3] = t.w;
        } else {
          sa.v[e][0] = ld(src);
        }
      }
#pragma unroll
      for (int e = 0; e < SB::SLOTS; ++e) {
        const int k = k0 + sb.line(e);
        sb.ok[e] = jin && k < K;
        const T* src = b_src(min(k, K - 1), nn, pp, jj);
        if constexpr (VEC) {
          float4 t;
          if constexpr (std::is_same<T, float>::value) t = ld4_dword_aligned(src);
          else t = ld4(src);
          sb.v[e][0] = t.x, sb.v[e][1] = t.y, sb.v[e][2] = t.z, sb.v[e][3] = t.w;
        } else {
          sb.v[e][0] = ld(src);
        }
      }
    } else if constexpr (VEC) {
      int nu = n, pu = p;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool in = j + u < je;
        const int nq = in ? nu : 0, pq = in ? pu : 0;
#pragma unroll
        for (int e = 0; e < SA::SLOTS; ++e) {
          const int m = i0 + sa.line(e);
          sa.ok[e] = m < M;
          const float t = ld(dy + ((int64_t)nq * M + min(m, M - 1)) * P + pq);
          sa.v[e][u] = in ? t : 0.f;
        }
#pragma unroll
        for (int e = 0; e < SB::SLOTS; ++e) {
          const int k = k0 + sb.line(e);
          sb.ok[e] = k < K;
          const float t = ld(b_src(min(k, K - 1), nq, pq, in ? j + u : 0));
          sb.v[e][u] = in ? t : 0.f;
        }
        if (++pu >= P) pu = 0, ++nu;
      }
    }
    j += BK;
    p += BK;
    while (p >= P) {
      p -= P;
      ++n;
    }
  };

  f32x16 acc[TM][TN];
  zero_acc<TM, TN>(acc);

  const int ktiles = (int)((je - js + BK - 1) / BK);
  if (ktiles > 0) {
    fetch();
    sa.store(As0);
    sb.store(Bs0);
  }
  __syncthreads();
  for (int kt = 0; kt < ktiles; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < ktiles) fetch();
    mma_slab<BM, BN, BK, TM, TN, true, true>(As0 + cur * LA::SIZE, Bs0 + cur * LB::SIZE, wm0, wn0, lane, acc);
    if (kt + 1 < ktiles) {
      sa.store(As0 + (cur ^ 1) * LA::SIZE);
      sb.store(Bs0 + (cur ^ 1) * LB::SIZE);
    }
    __syncthreads();
  }

  float* dst = out + (int64_t)blockIdx.y * M * K;
  const int l32 = lane & 31;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int k = k0 + wn0 + ni * 32 + l32;
    if (k >= K) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int m = i0 + wm0 + mi * 32 + acc_row(q, lane);
        if (m < M) dst[(int64_t)m * K + k] = acc[mi][ni][q];
      }
  }
}

static constexpr int kBfBK = 32;
static int bwd_filter_bm(const ConvGeom& g) { return g.M <= 32 ? 32 : (g.M <= 64 ? 64 : 128); }
// (a kernel matrix of at most 64 columns under 128-row tiles - the one-map layers' taps as columns - takes 64-column
// tiles: half the B operand to fetch and half the products)
static int bwd_filter_bn(const ConvGeom& g) { return g.K <= 64 && g.M > 64 ? 64 : 128; }

static int bwd_filter_chunk(const ConvGeom& g) {
  const int64_t tiles = ceil_div(g.M, bwd_filter_bm(g)) * ceil_div(g.K, bwd_filter_bn(g));
  int64_t want = 512 / tiles;
  // (a result of a few tiles only: shorter ranges, so that every compute unit still gets two blocks)
  const int64_t shortest = tiles <= 8 ? 256 : 512;
  const int64_t max_splits = g.N / shortest > 0 ? g.N / shortest : 1;
  if (want < 1) want = 1;
  if (want > max_splits) want = max_splits;
  int64_t chunk = ceil_div(g.N, want);
  chunk = ceil_div(chunk, kBfBK) * kBfBK;
  return (int)chunk;
}

int bwd_filter_splits(const ConvGeom& g) { return (int)ceil_div(g.N, bwd_filter_chunk(g)); }

size_t bwd_filter_partial_bytes(const ConvGeom& g) {
  const int splits = bwd_filter_splits(g);
  return splits > 1 ? (size_t)splits * g.M * g.K * sizeof(float) : 0;
}

template <int BM, int BN, int WM, int WN, bool VEC, typename T>
static void launch_bf_one(const ConvGeom& g, const void* dy, const void* col, const void* xin, float* out, int tiles_m,
                          int chunk, dim3 grid, hipStream_t st) {
  const size_t lds = gemm_lds_bytes<BM, BN, kBfBK, true, true>();
  auto kernel = bwd_filter_f32_kernel<BM, BN, kBfBK, WM, WN, VEC, T>;
  static bool opted_in = false;
  allow_lds(kernel, lds, opted_in);
  hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds, st, g, (const T*)dy, (const T*)col, (const T*)xin, out, tiles_m,
                     chunk);
}

template <int BM, int BN, int WM, int WN>
static void launch_bf(const ConvGeom& g, int dtype, const void* dy, const void* col, const void* xin, float* out,
                      int tiles_m, int chunk, dim3 grid, bool vec, hipStream_t st) {
  if (dtype == VCNN_BF16) {
    if (vec) launch_bf_one<BM, BN, WM, WN, true, bf16>(g, dy, col, xin, out, tiles_m, chunk, grid, st);
    else launch_bf_one<BM, BN, WM, WN, false, bf16>(g, dy, col, xin, out, tiles_m, chunk, grid, st);
  } else {
    if (vec) launch_bf_one<BM, BN, WM, WN, true, float>(g, dy, col, xin, out, tiles_m, chunk, grid, st);
    else launch_bf_one<BM, BN, WM, WN, false, float>(g, dy, col, xin, out, tiles_m, chunk, grid, st);
  }
}

vcnn_status launch_bwd_filter_gemm_f32(const ConvGeom& g, int dtype, const void* dy, const void* col, const void* xin,
                                       float* dw, float* partial, hipStream_t st) {
  const int chunk = bwd_filter_chunk(g);
  const int splits = bwd_filter_splits(g);
  float* out = splits > 1 ? partial : dw;
  const int bm = bwd_filter_bm(g);
  const int tiles_m = (int)ceil_div(g.M, bm);
  const int64_t tiles = (int64_t)tiles_m * ceil_div(g.K, bwd_filter_bn(g));
  const dim3 grid((unsigned)tiles, (unsigned)splits);
  if (splits > 65535) return fail(VCNN_ERR_UNSUPPORTED, "bwd_filter: too many contraction splits");
  const void* b = xin ? xin : col;
  // bf16: 8-byte loads need groups of four that keep the tensors' alignment; float: 16-byte loads at any dword
  const bool vec = dtype == VCNN_BF16 ? g.P % 4 == 0 && g.N % 4 == 0 && in_aligned(dy, dtype) && in_aligned(b, dtype)
                                      : g.P >= 4 && ((reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(b)) & 3) == 0;
  if (bm == 32)
    launch_bf<32, 128, 32, 32>(g, dtype, dy, col, xin, out, tiles_m, chunk, grid, vec, st);
  else if (bm == 64)
    launch_bf<64, 128, 32, 64>(g, dtype, dy, col, xin, out, tiles_m, chunk, grid, vec, st);
  else if (bwd_filter_bn(g) == 64)
    launch_bf<128, 64, 64, 32>(g, dtype, dy, col, xin, out, tiles_m, chunk, grid, vec, st);
  else
    launch_bf<128, 128, 64, 64>(g, dtype, dy, col, xin, out, tiles_m, chunk, grid, vec, st);
  vcnn_status s = check_launch("bwd_filter_f32");
  if (s != VCNN_OK || splits == 1) return s;
  return launch_sum_slices(partial, nullptr, dw, VCNN_F32, g.M * g.K, splits, 1, 1, 0, st);
}


// gw: dW(o, i) = sum_b dY[b][o] X[b][i] (A = dY read across rows, B = X), gx: dX(b, i) = sum_o dY[b][o] W[o][i]
// (A = dY contraction-contiguous, B = W); both must satisfy gemm_is_small.
vcnn_status launch_fc_bwd_small(const GemmArgs& gw, const GemmArgs& gx, hipStream_t st) {
  const int waves = std::max(small_waves(gw.K), small_waves(gx.K));
  const int tiles_w = (int)small_blocks(gw), tiles_x = (int)small_blocks(gx);
  const dim3 grid((unsigned)(tiles_w + tiles_x)), block(64 * waves);
  const size_t lds = (size_t)(waves - 1) * 16 * 64 * sizeof(float);
  const int tm_w = (int)ceil_div(gw.M, small_side(gw)), tm_x = (int)ceil_div(gx.M, small_side(gx));
  const int w16 = small_use16(gw), x16 = small_use16(gx);
  // each product keeps the split it has when launched alone (surplus waves get an empty share), so the fused
  // launch returns the same bits as two separate ones
  const int kp_w = small_kper(gw, small_waves(gw.K)), kp_x = small_kper(gx, small_waves(gx.K));
  const bool av = in_aligned(gx.A, gx.in_dtype) && gx.a_si % 4 == 0 && gx.K % 4 == 0;
  const int x_first = gx.K >= gw.K;
  if (gw.in_dtype == VCNN_BF16) {
    if (av) hipLaunchKernelGGL((fc_bwd_small_kernel<true, bf16>), grid, block, lds, st, gw, gx, tiles_w, tm_w, kp_w, tiles_x, tm_x, kp_x, x_first, w16, x16);
    else hipLaunchKernelGGL((fc_bwd_small_kernel<false, bf16>), grid, block, lds, st, gw, gx, tiles_w, tm_w, kp_w, tiles_x, tm_x, kp_x, x_first, w16, x16);
  } else {
    if (av) hipLaunchKernelGGL((fc_bwd_small_kernel<true, float>), grid, block, lds, st, gw, gx, tiles_w, tm_w, kp_w, tiles_x, tm_x, kp_x, x_first, w16, x16);
    else hipLaunchKernelGGL((fc_bwd_small_kernel<false, float>), grid, block, lds, st, gw, gx, tiles_w, tm_w, kp_w, tiles_x, tm_x, kp_x, x_first, w16, x16);
  }
  return check_launch("fc_bwd_small");
}

}  // namespace vcnn
