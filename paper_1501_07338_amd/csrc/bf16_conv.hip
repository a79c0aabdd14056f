// Implicit-unroll convolution of the bf16 variant on v_mfma_f32_32x32x16_bf16 (fp32 accumulate).
//
// As in the fp32 kernel the patch matrix phi_c(x) of Eq. 2 / Eq. 4 is never formed: a block stages the
// input rows its output pixels touch (with halo, zero padded) in LDS and reads the B operand of every
// MFMA at lane_base(pixel) + tap_offset.  What differs is how the two operands reach the matrix cores:
//
//  * The input is first re-laid channel-interleaved, x8[n][c/8][h][w][8] (one small pass over the
//    tensor), so that a halo position is one 16-byte word holding the 8 contraction elements a lane
//    feeds to one MFMA.  The halo tile is double buffered and filled with direct global->LDS loads
//    (global_load_lds_dwordx4: lane i of a wave deposits its 16 bytes at base + 16 i), issued for the
//    next chunk of channel groups before the MFMAs of the current one, so staging overlaps compute and
//    a chunk change costs one barrier.  Positions outside the image read a 16-byte block of zeros.
//  * The kernel matrix never goes through LDS.  It is re-ordered once per call into MFMA fragment order,
//    wf[row tile][chunk][step][lane][8]: the A operand of a step is one fully coalesced 1 KB read per
//    wave straight from L2 into registers, prefetched one slab (4 steps) ahead.  Without a shared A
//    slab the main loop has no barrier; blocks synchronise only when the halo tile changes.
//  * A wave owns 64 output maps x 32*TN pixels (LDS traffic per MFMA falls with the tile size).  The four
//    waves of a block either take different maps (many maps) or split the contraction between them (few
//    maps; partial sums are added in a fixed order through LDS at the end).
//
// Contraction order: (channel group of 8, r, s, channel in group); a step contracts two (group, tap)
// pairs, lanes 0-31 the even one and lanes 32-63 the odd one.  Layers with 33..48 output maps (M16) run on
// v_mfma_f32_16x16x32_bf16 instead - three 16-row tiles per wave rather than 64 rows a quarter of which is
// padding; there a step contracts four pairs, lanes 16 k .. 16 k + 15 the k-th of them.  The input gradient is the same kernel
// run on dy with the flipped, transposed kernels (the re-ordering pass does the flip).
#include <algorithm>
#include <type_traits>

#include "bf16_core.h"
#include "common.h"
#include "elem.h"

namespace vcnn {

static constexpr int kThreads = 256;
static constexpr size_t kLdsBudget = 78 * 1024;  // two blocks per CU

// x8[n][g][pos][c8] = x[n][8g + c8][pos], zero for channels >= C; x8[total] = 0 (the padding source)
__global__ __launch_bounds__(kThreads) void interleave_channels_kernel(const bf16* __restrict__ x, uint4* __restrict__ x8,
                                                                       int C, int CG, int HW, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i == 0) x8[total] = make_uint4(0u, 0u, 0u, 0u);
  if (i >= total) return;
  const int pos = (int)(i % HW);
  const int64_t t = i / HW;
  const int g = (int)(t % CG);
  const int64_t n = t / CG;
  const bf16* src = x + (n * C + g * 8) * HW + pos;
  uint32_t v[8];
#pragma unroll
  for (int c8 = 0; c8 < 8; ++c8) {
    const bool ok = g * 8 + c8 < C;
    const uint16_t b = src[ok ? (int64_t)c8 * HW : 0].bits;
    v[c8] = ok ? b : 0u;
  }
  x8[i] = make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
}

// wf[mt][ch][jl][lane][c8] = w(row = 32 mt + lane % 32, channel = 8 (ch*cgc + gl) + c8, tap q) where
// (gl, q) = divmod(2 jl + lane / 32, RS); zero outside the matrix or the chunk.  With m16: row = 16 mt + lane % 16
// and (gl, q) = divmod(4 jl + lane / 16, RS).
// w(row, channel, q) = in[row*so + channel*si + (flip ? RS-1-q : q)].
__global__ __launch_bounds__(kThreads) void reorder_weights_frag_kernel(const bf16* __restrict__ in, bf16* __restrict__ out,
                                                                        int CO, int CI, int RS, int64_t so, int64_t si,
                                                                        int flip, int cgc, int nchunks, int steps,
                                                                        int m16, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= total) return;
  const int c8 = (int)(i & 7);
  const int lane = (int)(i >> 3) & 63;
  int64_t t = i >> 9;
  const int jl = (int)(t % steps);
  t /= steps;
  const int ch = (int)(t % nchunks);
  const int mt = (int)(t / nchunks);
  const int row = m16 ? mt * 16 + (lane & 15) : mt * 32 + (lane & 31);
  const int u = m16 ? 4 * jl + (lane >> 4) : 2 * jl + (lane >> 5);
  const int gl = u / RS, q = u - gl * RS;
  const int c = (ch * cgc + gl) * 8 + c8;
  bf16 v;
  v.bits = 0;
  if (row < CO && gl < cgc && c < CI) v = in[(int64_t)row * so + (int64_t)c * si + (flip ? RS - 1 - q : q)];
  out[i] = v;
}

// The same re-ordering, eight taps per thread, for kernels whose tap count and strides are multiples of eight (and whose
// matrix is 16-byte aligned): a thread reads the 8 consecutive taps of one (row, channel) as one 16-byte word - the
// element-wise form reads 2 bytes per thread at strides of a kernel's size - and stores them to the 8 (group, tap) pairs
// they belong to.  Threads are ordered (channel in group, row in tile) fastest, so that the 2-byte stores of one tap
// fill 128 contiguous bytes per 8 rows.  Entries outside the matrix or the chunk are written as zeros, as above.
__global__ __launch_bounds__(kThreads) void reorder_weights_frag8_kernel(const bf16* __restrict__ in, bf16* __restrict__ out,
                                                                         int CO, int CI, int RS, int64_t so, int64_t si,
                                                                         int flip, int cgc, int nchunks, int uch, int m16,
                                                                         int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= total) return;
  const int T = m16 ? 16 : 32;
  const int c8 = (int)(i & 7);
  int64_t t = i >> 3;
  const int rt = (int)(t % T);
  t /= T;
  const int ub = (int)(t % (uch / 8));
  t /= uch / 8;
  const int ch = (int)(t % nchunks);
  const int mt = (int)(t / nchunks);
  const int row = mt * T + rt;
  const int u0 = ub * 8;
  const int gl = u0 / RS, q0 = u0 - gl * RS;
  const int c = (ch * cgc + gl) * 8 + c8;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (row < CO && gl < cgc && c < CI)
    v = *reinterpret_cast<const uint4*>(in + (int64_t)row * so + (int64_t)c * si + (flip ? RS - 8 - q0 : q0));
  const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
  const int steps = uch / 8 * (m16 ? 2 : 4);
  bf16* const dst = out + ((int64_t)mt * nchunks + ch) * steps * 512 + c8;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int e = flip ? 7 - k : k;  // position of tap q0 + k inside the word
    bf16 b;
    b.bits = (uint16_t)(w4[e >> 1] >> (16 * (e & 1)));
    const int u = u0 + k;
    const int jl = m16 ? u >> 2 : u >> 1;
    const int lane = m16 ? (u & 3) * 16 + rt : (u & 1) * 32 + rt;
    dst[((int64_t)jl * 64 + lane) * 8] = b;
  }
}

struct HaloBf16Args {
  const uint4* x8;    // [n][cg][h][w] positions of 8 channels
  int64_t x8_term;    // TERMS > 1: distance between the terms of x8, and of wf, in 16-byte words
  int64_t wf_term;
  const uint4* zero;  // 16 zero bytes
  const uint4* wf;    // [mt][chunk][step][64 lanes] fragments
  const float* bias;  // [m] or null
  bf16* y;            // [n][m][oh][ow]
  float* y32;         // not null: the result goes here instead, in float, added to what is there when `accumulate`
  int accumulate;
  int n, h, w, m, r, s, ph, pw, oh, ow, P;
  int tiles_m, tiles_per_img;
  int cg, cgc, nchunks;
  int nr, wp;         // halo rows and row pitch (positions) per group
  int uch;            // (group, tap) pairs per chunk, padded to a multiple of 8
  int hpos;           // positions per halo buffer (cgc*nr*wp rounded up to a multiple of 64)
  int nbuf;           // halo buffers: 2 = the next chunk is staged during the products of this one, 1 = between chunks
  int relu;
};

// TERMS = 3: both operands are given as three bfloat16 terms each (a float split exactly into three), and a step
// multiplies the six largest of the nine term pairs - smallest first - into the same accumulators: the float product
// to within float rounding, with every staged word and every fragment used for two or three MFMAs instead of one.
template <int WAVES_M, int WAVES_K, int TM, int TN, bool M16 = false, int WAVES_N = 1, int TERMS = 1>
__global__ __launch_bounds__(kThreads, 2) void conv_halo_bf16_kernel(HaloBf16Args a) {
  static_assert(TERMS == 1 || TERMS == 3, "plain bfloat16 operands, or floats as three terms");
  constexpr int PAIRS = TERMS == 1 ? 1 : 6;
  constexpr int kTermA[6] = {2, 0, 1, 1, 0, 0}, kTermB[6] = {0, 2, 1, 0, 1, 0};  // kernel-matrix term, input term
  static_assert(WAVES_M * WAVES_K * WAVES_N * 64 == kThreads, "four waves per block");
  static_assert(!M16 || WAVES_M == 1, "16-row tiles: every wave holds all rows");
  constexpr int TILE = M16 ? 16 : 32;     // rows and pixels of one accumulator tile
  constexpr int AQ = M16 ? 4 : 16;        // accumulator registers per tile
  constexpr int SPS = M16 ? 2 : 4;        // MFMA steps per slab of 8 (group, tap) pairs
  using Acc = typename std::conditional<M16, f32x4, f32x16>::type;
  constexpr int BM = TILE * TM * WAVES_M, WN = TILE * TN, BN = WN * WAVES_N;  // block rows, wave pixels, block pixels
  extern __shared__ uint4 smem16[];
  int* const tbl = reinterpret_cast<int*>(smem16);  // [uch], per slab of 8 pairs: [half][4]
  int* const nxt = tbl + a.uch;                     // [uch/8 + 4]: next slab with work, first such slab per wave
  uint4* const hbuf = smem16 + a.uch / 4 + (a.uch / 8 + 7) / 4;  // nbuf x TERMS x [cgc][nr][wp], each padded to hpos positions

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lcol = lane & (TILE - 1), half = lane / TILE;  // tile column / row of this lane, its pair of the step
  const int wave_m = wave % WAVES_M, wave_k = (wave / WAVES_M) % WAVES_K, wave_n = wave / (WAVES_M * WAVES_K);
  const int pw0 = wave_n * WN;  // first pixel of this wave inside the block's tile
  const int tm = blockIdx.x % a.tiles_m;
  const int tj = blockIdx.x / a.tiles_m;
  const int n = tj / a.tiles_per_img;
  const int p0 = (tj - n * a.tiles_per_img) * BN;
  const int i0 = tm * BM + wave_m * TILE * TM;  // first output map of this wave
  const int RS = a.r * a.s;
  const int plane = a.nr * a.wp;
  const int oh_first = p0 / a.ow;

  // table: position offset of pair u = (group gl, tap q) inside the halo tile; padding pairs point at 0
  // (their kernel-matrix entries are zero).  Entry u = 8*sl + 2*i + h is stored at 8*sl + 4*h + i (M16: entry
  // 8*sl + 4*i + h at 8*sl + 2*h + i), so a lane reads the offsets of all its steps of a slab as one vector.
  for (int u = tid; u < a.uch; u += kThreads) {
    int off = 0;
    if (u < a.cgc * RS) {
      const int gl = u / RS;
      const int q = u - gl * RS;
      const int r = q / a.s;
      off = gl * plane + r * a.wp + (q - r * a.s);
    }
    const int sl = u >> 3, w8 = u & 7;
    tbl[sl * 8 + (M16 ? (w8 & 3) * 2 + (w8 >> 2) : (w8 & 1) * 4 + (w8 >> 1))] = off;
  }

  int lane_base[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = min(p0 + pw0 + ni * TILE + lcol, a.P - 1);
    const int oh = p / a.ow;
    lane_base[ni] = (oh - oh_first) * a.wp + (p - oh * a.ow);
  }

  // Slabs whose 8 (group, tap) pairs all lie on kernel rows that meet only the zero border for every
  // output row of this tile contribute nothing (the input gradient of a 'valid' layer is a fully padded
  // correlation, where this is a quarter of the work).  nxt[sl] = next slab of the same wave that has
  // work (>= uch/8: none), nxt[uch/8 + k] = first such slab of wave k.
  {
    const int chunk_slabs = a.uch / 8;
    const int oh_last = min(p0 + BN - 1, a.P - 1) / a.ow;
    const int r_lo = a.ph - oh_last, r_hi = a.h - 1 + a.ph - oh_first;  // kernel rows that reach the image
    auto has_work = [&](int sl) {
      const int u0 = sl * 8, u1 = min(u0 + 7, a.cgc * RS - 1);
      if (u0 > u1) return false;  // padding slab
      const int g0 = u0 / RS, g1 = u1 / RS;
      if (g0 != g1) return true;
      const int r0 = (u0 - g0 * RS) / a.s, r1 = (u1 - g0 * RS) / a.s;
      return r1 >= r_lo && r0 <= r_hi;
    };
    for (int sl = tid; sl < chunk_slabs + WAVES_K; sl += kThreads) {
      int t = sl < chunk_slabs ? sl + WAVES_K : sl - chunk_slabs;
      while (t < chunk_slabs && !has_work(t)) t += WAVES_K;
      nxt[sl] = min(t, chunk_slabs);
    }
  }

  Acc acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < AQ; ++q) acc[mi][ni][q] = 0.f;

  const uint4* x8n = a.x8 + (int64_t)n * a.cg * a.h * a.w;
  const int steps = a.uch / 8 * SPS;                         // fragment steps per chunk
  const int chunk_slabs = a.uch / 8;
  const int64_t mstride = (int64_t)a.nchunks * steps * 64;   // fragments per row tile
  const uint4* wf0 = a.wf + (int64_t)(i0 / TILE) * mstride + lane;

  // A fragments of the slab this wave works on next: af[step in slab][row tile]
  // (three terms: one step ahead instead of one slab - a step is 6 * TM * TN MFMAs long - which leaves the registers
  // for reading the halo words a step ahead as well)
  constexpr int AHEAD = TERMS == 3 ? 1 : SPS;
  uint4 af[TERMS][AHEAD][TM];
  auto load_a = [&](int ch, int sl) {
    const uint4* src = wf0 + ((int64_t)ch * steps + sl * SPS) * 64;
#pragma unroll
    for (int t = 0; t < TERMS; ++t)
#pragma unroll
      for (int i = 0; i < AHEAD; ++i)
#pragma unroll
        for (int mi = 0; mi < TM; ++mi) af[t][i][mi] = src[t * a.wf_term + mi * mstride + i * 64];
  };
  __syncthreads();  // nxt is complete
  const int first_work = nxt[chunk_slabs + wave_k];  // this wave's first slab with work in any chunk
  const int first_sl = min(first_work, chunk_slabs - 1);
  load_a(0, first_sl);

  // Asynchronous halo staging: positions in flat tile order, 64 consecutive positions per wave and
  // load instruction; the walk (rx, ry, gl) is the same for every chunk.
  const int dq = kThreads / a.wp, dr = kThreads - dq * a.wp;
  const int row_s = tid / a.wp, rx_s = tid - row_s * a.wp;
  const int gl_s = row_s / a.nr, ry_s = row_s - gl_s * a.nr;
  auto stage = [&](int ch, uint4* dst) {
    // every chunk fills the whole tile: groups beyond the last one become zeros, because the padding
    // pairs of a short last chunk still read their positions (times zero weights)
    const int g0 = ch * a.cgc;
    const int npos = a.cgc * plane;
    int rx = rx_s, ry = ry_s, gl = gl_s;
    for (int b0 = wave * 64; b0 < npos; b0 += kThreads) {  // b0: first position of this wave's 64 (uniform)
      const int ih = oh_first - a.ph + ry, iw = rx - a.pw;
      const bool ok = b0 + lane < npos && g0 + gl < a.cg && ih >= 0 && ih < a.h && iw >= 0 && iw < a.w;
      const uint4* src = ok ? x8n + ((g0 + gl) * a.h + ih) * a.w + iw : a.zero;
#pragma unroll
      for (int t = 0; t < TERMS; ++t) load_to_lds16(ok ? src + t * a.x8_term : src, dst + t * a.hpos + b0);
      rx += dr;
      ry += dq;
      if (rx >= a.wp) rx -= a.wp, ++ry;
      while (ry >= a.nr) ry -= a.nr, ++gl;
    }
  };
  stage(0, hbuf);
  constexpr int kBuf = TERMS;  // planes per halo buffer

  for (int ch = 0; ch < a.nchunks; ++ch) {
    const int ulen = min(a.cgc, a.cg - ch * a.cgc) * RS;  // valid (group, tap) pairs in this chunk
    const int slabs = (ulen + 7) >> 3;
    const uint4* halo = hbuf + (ch & (a.nbuf - 1)) * kBuf * a.hpos;
    // this chunk's tile has landed (every wave waits for its own loads, the barrier publishes them) and
    // every wave is done with the other buffer (first pass: the table is complete)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    if (a.nbuf == 2 && ch + 1 < a.nchunks) stage(ch + 1, hbuf + ((ch + 1) & 1) * kBuf * a.hpos);

    if constexpr (TERMS == 3) {
      // Both operands of a step are requested a step ahead: the halo words of step i + 1 (LDS) and the fragments of
      // step i + 1 (second-level cache) are on their way while the 6 * TM * TN MFMAs of step i run, so that the two
      // waves of a SIMD never wait for LDS at the same time.  Only the first step of a chunk waits for its words.
      auto read_offsets = [&](int sl, int (&dst)[4]) {
        const int4 o4 = *reinterpret_cast<const int4*>(tbl + sl * 8 + half * 4);
        dst[0] = o4.x, dst[1] = o4.y, dst[2] = o4.z, dst[3] = o4.w;
      };
      int o[4] = {0, 0, 0, 0};
      uint4 bfr[TERMS][TN];
      if (first_work < slabs) {
        read_offsets(first_work, o);
#pragma unroll
        for (int t = 0; t < TERMS; ++t)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni) bfr[t][ni] = halo[t * a.hpos + lane_base[ni] + o[0]];
      }
      for (int sl = first_work; sl < slabs;) {
        const int after = nxt[sl];
        int nch = ch, nsl = after;
        if (nsl >= slabs) {
          if (ch + 1 < a.nchunks) nch = ch + 1, nsl = first_sl;
          else nsl = sl;
        }
        const uint4* csrc = wf0 + ((int64_t)ch * steps + sl * SPS) * 64;
        const uint4* nsrc = wf0 + ((int64_t)nch * steps + nsl * SPS) * 64;
        // offsets of the slab after this one (past the chunk's last slab: any slab's - the words read with them are
        // dropped when the next chunk reads its own first step)
        int on[4];
        read_offsets(min(after, chunk_slabs - 1), on);
#pragma unroll
        for (int i = 0; i < SPS; ++i) {
          uint4 cur[TERMS][TM], bnext[TERMS][TN];
          const uint4* nptr = i + 1 < SPS ? csrc + (i + 1) * 64 : nsrc;
          const int onext = i + 1 < SPS ? o[(i + 1) & 3] : on[0];
          // (requested in the order the next step's MFMAs first use them, so that its first MFMA waits for the
          // oldest request only, not for all of them)
          constexpr int kOrderA[3] = {2, 0, 1}, kOrderB[3] = {0, 2, 1};
#pragma unroll
          for (int k = 0; k < TERMS; ++k)
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) {
              const int t = kOrderA[k];
              cur[t][mi] = af[t][0][mi];
              af[t][0][mi] = nptr[t * a.wf_term + mi * mstride];
            }
#pragma unroll
          for (int k = 0; k < TERMS; ++k)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
              const int t = kOrderB[k];
              bnext[t][ni] = halo[t * a.hpos + lane_base[ni] + onext];
            }
#pragma unroll
          for (int pr = 0; pr < PAIRS; ++pr)
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
              for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(cur[kTermA[pr]][mi], bfr[kTermB[pr]][ni], acc[mi][ni]);
          // issue order of the step: the requests of the next step go out between this step's MFMAs, one fragment
          // load and one halo read after every TM * TN of them, in the shadow of the matrix pipe
#pragma unroll
          for (int k = 0; k < TERMS * TM; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, PAIRS * TN / TERMS, 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                   // global read
            if (k < TERMS * TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
          }
#pragma unroll
          for (int t = 0; t < TERMS; ++t)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) bfr[t][ni] = bnext[t][ni];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = on[i];
        sl = after;
      }
    } else {
      // bfloat16 operands: the fragments are requested a slab ahead (a step is only TM * TN MFMAs long), the halo words
      // a step ahead, both between the MFMAs of the current step
      auto read_offsets = [&](int sl, int (&dst)[4]) {
        if (M16) {
          const int2 o2 = *reinterpret_cast<const int2*>(tbl + sl * 8 + half * 2);
          dst[0] = o2.x, dst[1] = o2.y, dst[2] = 0, dst[3] = 0;
        } else {
          const int4 o4 = *reinterpret_cast<const int4*>(tbl + sl * 8 + half * 4);
          dst[0] = o4.x, dst[1] = o4.y, dst[2] = o4.z, dst[3] = o4.w;
        }
      };
      int o[4] = {0, 0, 0, 0};
      uint4 bfr[TN];
      if (first_work < slabs) {
        read_offsets(first_work, o);
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) bfr[ni] = halo[lane_base[ni] + o[0]];
      }
      for (int sl = first_work; sl < slabs;) {
        // where this wave continues: its next slab with work in this chunk, else its first one in the next
        // chunk (the fragment loads do not depend on the halo tile, so they stay in flight across the change)
        const int after = nxt[sl];
        int nch = ch, nsl = after;
        if (nsl >= slabs) {
          if (ch + 1 < a.nchunks) nch = ch + 1, nsl = first_sl;
          else nsl = sl;
        }
        const uint4* nsrc = wf0 + ((int64_t)nch * steps + nsl * SPS) * 64;
        // offsets of the slab after this one (past the chunk's last slab: any slab's - the words read with them are
        // dropped when the next chunk reads its own first step)
        int on[4];
        read_offsets(min(after, chunk_slabs - 1), on);
#pragma unroll
        for (int i = 0; i < SPS; ++i) {
          uint4 cur[TM], bnext[TN];
          const int onext = i + 1 < SPS ? o[(i + 1) & 3] : on[0];
#pragma unroll
          for (int mi = 0; mi < TM; ++mi) {
            cur[mi] = af[0][i][mi];
            af[0][i][mi] = nsrc[mi * mstride + i * 64];
          }
#pragma unroll
          for (int ni = 0; ni < TN; ++ni) bnext[ni] = halo[lane_base[ni] + onext];
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(cur[mi], bfr[ni], acc[mi][ni]);
          // issue order: one halo read (and, while there are any, one fragment load) after every TM MFMAs
#pragma unroll
          for (int k = 0; k < TN; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, TM, 0);              // MFMA
            if (k < TM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // global read
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);              // LDS read
          }
#pragma unroll
          for (int ni = 0; ni < TN; ++ni) bfr[ni] = bnext[ni];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = on[i];
        sl = after;
      }
    }
    if (a.nbuf == 1 && ch + 1 < a.nchunks) {  // one buffer: every wave is done reading it, then it is refilled
      __syncthreads();
      stage(ch + 1, hbuf);
    }
  }

  // contraction split between waves: add the partial sums in wave order through LDS
  if (WAVES_K > 1) {
    float* red = reinterpret_cast<float*>(smem16);  // [TM*TN*AQ][64 lanes]
#pragma unroll 1
    for (int k = 1; k < WAVES_K; ++k) {
      __syncthreads();
      if (wave_k == k) {
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int q = 0; q < AQ; ++q) red[(((wave_m * TM + mi) * TN + ni) * AQ + q) * 64 + lane] = acc[mi][ni][q];
      }
      __syncthreads();
      if (wave_k == 0) {
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int q = 0; q < AQ; ++q) acc[mi][ni][q] += red[(((wave_m * TM + mi) * TN + ni) * AQ + q) * 64 + lane];
      }
    }
    if (wave_k != 0) return;
  }

#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int p = p0 + pw0 + ni * TILE + lcol;
    if (p >= a.P) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < AQ; ++q) {
        // result tile: 32 x 32 -> row 8*(q/4) + 4*(lane/32) + q%4; 16 x 16 -> row 4*(lane/16) + q; column = lcol
        const int i = i0 + mi * TILE + (M16 ? 4 * half + q : 8 * (q >> 2) + 4 * half + (q & 3));
        if (i < a.m) {
          float v = acc[mi][ni][q];
          const int64_t at = ((int64_t)n * a.m + i) * a.P + p;
          if (a.y32 && a.accumulate) v += a.y32[at];
          if (a.bias) v += a.bias[i];
          if (a.relu) v = fmaxf(v, 0.f);
          if (a.y32) a.y32[at] = v;
          else st(a.y + at, v);
        }
      }
  }
}

// ---- planning ---------------------------------------------------------------------------------------------
static constexpr int kTnChoices[] = {2, 4, 5};     // 32-pixel tiles per wave
static constexpr int kTn16Choices[] = {4, 8, 10};  // 16-pixel tiles per wave (the same pixel counts)

// One arrangement of the four waves (waves_m along the maps, waves_n along the pixels, the rest along the contraction);
// *cost_out is the estimated time in units of one 32-pixel wave tile.
static bool plan_arrangement(int waves_m, int waves_n, int n, int c, int h, int w, int m, int r, int s, int ph, int pw,
                             HaloBf16Plan* p, double* cost_out, int terms, int nbuf = 2) {
  const int oh = h + 2 * ph - r + 1, ow = w + 2 * pw - s + 1;
  if (oh <= 0 || ow <= 0) return false;
  const int rs = r * s;
  const int cg = (c + 7) / 8;
  if ((int64_t)cg * h * w > 0x7fffffffLL) return false;  // 32-bit position offsets inside a sample
  p->m16 = m > 32 && m <= 48;  // three 16-row tiles instead of two 32-row ones
  p->waves_m = waves_m, p->waves_n = waves_n, p->terms = terms, p->nbuf = nbuf;
  p->tm = p->m16 ? 3 : (m <= 32 ? 1 : 2);  // row tiles per wave
  const int tile = p->m16 ? 16 : 32, aq = p->m16 ? 4 : 16, sps = p->m16 ? 2 : 4;
  const int waves_k = 4 / (p->waves_m * p->waves_n);
  const int bm = tile * p->tm * p->waves_m;
  const int tiles_m = (int)ceil_div(m, bm);
  const int wp = w + 2 * pw;
  // pixel tile: fewest rounds of 512 resident blocks, weighted by the tile width (time per tile)
  const int64_t P = (int64_t)oh * ow;
  int best_tn = 0, best_cgc = 0, best_nr = 0;
  double best_cost = 0;
  // (three terms: the fragments and halo words of a step take three times the registers, which leaves room for the
  // accumulators of 64-pixel wave tiles only; their six products per step give those the reuse of wider tiles)
  for (int k = 0; k < (terms == 3 ? 1 : 3); ++k) {
    const int tn = p->m16 ? kTn16Choices[k] : kTnChoices[k];
    const int bn = tile * tn * p->waves_n;
    int rows = (bn + ow - 2) / ow + 1;
    if (rows > oh) rows = oh;
    const int nr = rows + r - 1;
    const size_t red_bytes = waves_k > 1 ? (size_t)p->waves_m * p->tm * tn * aq * 64 * sizeof(float) : 0;
    if (red_bytes > kLdsBudget) continue;
    int cgc = 0;
    for (int t = 1; t <= cg; ++t) {
      const int uch = (int)ceil_div((int64_t)t * rs, 8) * 8;
      const size_t hpos = ((size_t)t * nr * wp + 63) & ~(size_t)63;
      if ((size_t)uch * 4 + ((size_t)uch / 8 + 7) / 4 * 16 + nbuf * terms * hpos * 16 > kLdsBudget || uch > 4096) break;
      cgc = t;
    }
    if (cgc == 0) continue;
    const int64_t tiles = (int64_t)tiles_m * n * ceil_div(P, bn);
    if (tiles > 0x7fffffffLL) continue;
    const double wide = tile * tn / 32.0;
    const double cost = (double)ceil_div(tiles, 512) * wide * (1.0 + 0.5 / wide);  // wider tiles reuse A fragments better
    if (best_tn == 0 || cost < best_cost - 1e-9) best_tn = tn, best_cgc = cgc, best_nr = nr, best_cost = cost;
  }
  if (best_tn == 0) return false;
  // among chunk sizes at least half the largest, take the one that pads the fewest (group, tap) pairs
  int pick = best_cgc;
  double pick_waste = 2.0;
  for (int t = best_cgc; t >= 1 && 2 * t > best_cgc; --t) {
    const int64_t chunks = ceil_div(cg, t);
    const int last = cg - (int)(chunks - 1) * t;
    const int64_t slabs = (chunks - 1) * ceil_div((int64_t)t * rs, 8) + ceil_div((int64_t)last * rs, 8);
    const double waste = 1.0 - (double)cg * rs / (double)(slabs * 8);
    if (waste < pick_waste - 1e-9) pick = t, pick_waste = waste;
  }
  p->tn = best_tn, p->cg = cg, p->cgc = pick, p->nchunks = (int)ceil_div(cg, pick), p->nr = best_nr, p->wp = wp;
  p->uch = (int)ceil_div((int64_t)pick * rs, 8) * 8;
  const size_t red_bytes = waves_k > 1 ? (size_t)p->waves_m * p->tm * best_tn * aq * 64 * sizeof(float) : 0;
  p->hpos = (int)(((size_t)pick * best_nr * wp + 63) & ~(size_t)63);
  p->lds_bytes = std::max((size_t)p->uch * 4 + ((size_t)p->uch / 8 + 7) / 4 * 16 + nbuf * terms * (size_t)p->hpos * 16, red_bytes);
  p->x8_bytes = (((size_t)n * cg * h * w + 1) * 16 + 255) & ~(size_t)255;  // + the block of zeros
  p->wf_bytes = ((size_t)tiles_m * (bm / tile) * p->nchunks * (p->uch / 8 * sps) * 64 * 16 + 255) & ~(size_t)255;
  *cost_out = best_cost;
  return true;
}

bool conv_halo_bf16_plan(int n, int c, int h, int w, int m, int r, int s, int ph, int pw, HaloBf16Plan* p, int terms) {
  double cost = 0;
  if (terms != 1 && m <= 128) return false;  // the three-term form is built for the arrangements of many maps only
  if (m <= 128) return plan_arrangement(m > 64 ? 2 : 1, 1, n, c, h, w, m, r, s, ph, pw, p, &cost, terms);
  // many maps: the four waves take different maps of the same pixels, or - when the image is large enough for
  // four times as many pixels per block - different pixels of the same maps; these read the same kernel-matrix
  // fragments at about the same time, three of four from the first-level cache (cfg5 c3 forward: 0.8 instead
  // of 2.7 GB from the second level)
  HaloBf16Plan wide{};
  double wide_cost = 0;
  // (three halo planes of a large kernel may only fit LDS once: then a chunk is staged between the products of two
  // chunks, not during them, and the other resident block covers the gap)
  bool maps_ok = plan_arrangement(4, 1, n, c, h, w, m, r, s, ph, pw, p, &cost, terms);
  bool wide_ok = plan_arrangement(1, 4, n, c, h, w, m, r, s, ph, pw, &wide, &wide_cost, terms);
  if (terms == 3 && !maps_ok && !wide_ok) {
    maps_ok = plan_arrangement(4, 1, n, c, h, w, m, r, s, ph, pw, p, &cost, terms, 1);
    wide_ok = plan_arrangement(1, 4, n, c, h, w, m, r, s, ph, pw, &wide, &wide_cost, terms, 1);
  }
  if (wide_ok && (!maps_ok || wide_cost <= cost + 1e-9)) *p = wide;
  return maps_ok || wide_ok;
}

template <int WAVES_M, int WAVES_K, int TM, int TN, bool M16 = false, int WAVES_N = 1, int TERMS = 1>
static void launch_one(const HaloBf16Args& a, size_t lds, hipStream_t st) {
  const dim3 grid((unsigned)((int64_t)a.tiles_m * a.n * a.tiles_per_img)), block(kThreads);
  auto kernel = conv_halo_bf16_kernel<WAVES_M, WAVES_K, TM, TN, M16, WAVES_N, TERMS>;
  static bool opted = false;  // one flag per instantiation, i.e. per kernel
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsBudget);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, grid, block, lds, st, a);
}

template <int TN>
static void launch_tn(const HaloBf16Args& a, int waves_m, int waves_n, int tm, int terms, size_t lds, hipStream_t st) {
  if (terms == 3) {  // (planned for the two arrangements of many maps and 64-pixel wave tiles only)
    if constexpr (TN == 2) {
      if (waves_n == 4) launch_one<1, 1, 2, TN, false, 4, 3>(a, lds, st);
      else launch_one<4, 1, 2, TN, false, 1, 3>(a, lds, st);
    }
  } else if (waves_n == 4) launch_one<1, 1, 2, TN, false, 4>(a, lds, st);
  else if (waves_m == 4) launch_one<4, 1, 2, TN>(a, lds, st);
  else if (waves_m == 2) launch_one<2, 2, 2, TN>(a, lds, st);
  else if (tm == 2) launch_one<1, 4, 2, TN>(a, lds, st);
  else launch_one<1, 4, 1, TN>(a, lds, st);
}

vcnn_status launch_conv_halo_bf16(const HaloBf16Plan& p, int n, int c, int h, int w, int m, int r, int s, int ph, int pw,
                                  const void* x, const void* wgt, int64_t w_so, int64_t w_si, int flip, const float* bias,
                                  void* y, int relu, void* workspace, hipStream_t st, float* y32, int accumulate) {
  return launch_conv_halo_bf16_prepared(p, n, c, h, w, m, r, s, ph, pw, x, wgt, w_so, w_si, flip, bias, y, relu, workspace,
                                        (char*)workspace + p.x8_bytes, st, y32, accumulate);
}

// the two re-laying passes of one operand each, and the product on re-laid operands
static vcnn_status relay_input(const HaloBf16Plan& p, int n, int c, int h, int w, const void* x, void* x8_buf, hipStream_t st) {
  const int64_t total = (int64_t)n * p.cg * h * w;
  hipLaunchKernelGGL(interleave_channels_kernel, dim3((unsigned)ceil_div(total, kThreads)), dim3(kThreads), 0, st,
                     (const bf16*)x, (uint4*)x8_buf, c, p.cg, h * w, total);
  return check_launch("interleave_channels");
}

static vcnn_status relay_kernels(const HaloBf16Plan& p, int c, int m, int rs, const void* wgt, int64_t w_so, int64_t w_si,
                                 int flip, void* wf_buf, hipStream_t st) {
  const int tile = p.m16 ? 16 : 32;
  const int bm = tile * p.tm * p.waves_m;
  const int tiles_m = (int)ceil_div(m, bm);
  const int steps = p.uch / 8 * (p.m16 ? 2 : 4);
  const int64_t total = (int64_t)tiles_m * (bm / tile) * p.nchunks * steps * 512;
  if (rs % 8 == 0 && w_so % 8 == 0 && w_si % 8 == 0 && (reinterpret_cast<uintptr_t>(wgt) & 15) == 0) {
    const int64_t threads = (int64_t)tiles_m * (bm / tile) * p.nchunks * (p.uch / 8) * tile * 8;
    hipLaunchKernelGGL(reorder_weights_frag8_kernel, dim3((unsigned)ceil_div(threads, kThreads)), dim3(kThreads), 0, st,
                       (const bf16*)wgt, (bf16*)wf_buf, m, c, rs, w_so, w_si, flip, p.cgc, p.nchunks, p.uch, p.m16, threads);
    return check_launch("reorder_weights_frag8");
  }
  hipLaunchKernelGGL(reorder_weights_frag_kernel, dim3((unsigned)ceil_div(total, kThreads)), dim3(kThreads), 0, st,
                     (const bf16*)wgt, (bf16*)wf_buf, m, c, rs, w_so, w_si, flip, p.cgc, p.nchunks, steps, p.m16, total);
  return check_launch("reorder_weights_frag");
}

static vcnn_status launch_product(const HaloBf16Plan& p, int n, int h, int w, int m, int r, int s, int ph, int pw,
                                  const float* bias, void* y, int relu, const void* x8_buf, const void* wf_buf,
                                  hipStream_t st, float* y32, int accumulate) {
  const uint4* x8 = (const uint4*)x8_buf;
  const int tile = p.m16 ? 16 : 32;
  const int bm = tile * p.tm * p.waves_m;
  HaloBf16Args a{};
  a.x8 = x8, a.zero = x8 + (int64_t)n * p.cg * h * w, a.wf = (const uint4*)wf_buf, a.bias = bias, a.y = (bf16*)y;
  a.x8_term = (int64_t)(p.x8_bytes / 16), a.wf_term = (int64_t)(p.wf_bytes / 16);  // (read by the three-term form only)
  a.y32 = y32, a.accumulate = accumulate;
  a.n = n, a.h = h, a.w = w, a.m = m, a.r = r, a.s = s, a.ph = ph, a.pw = pw;
  a.oh = h + 2 * ph - r + 1, a.ow = w + 2 * pw - s + 1;
  a.P = a.oh * a.ow;
  a.tiles_m = (int)ceil_div(m, bm);
  a.tiles_per_img = (int)ceil_div(a.P, tile * p.tn * p.waves_n);
  a.cg = p.cg, a.cgc = p.cgc, a.nchunks = p.nchunks, a.nr = p.nr, a.wp = p.wp, a.uch = p.uch, a.hpos = p.hpos, a.relu = relu;
  a.nbuf = p.nbuf;
  if (p.m16) {
    if (p.tn == 4) launch_one<1, 4, 3, 4, true>(a, p.lds_bytes, st);
    else if (p.tn == 8) launch_one<1, 4, 3, 8, true>(a, p.lds_bytes, st);
    else launch_one<1, 4, 3, 10, true>(a, p.lds_bytes, st);
  } else if (p.tn == 2) launch_tn<2>(a, p.waves_m, p.waves_n, p.tm, p.terms, p.lds_bytes, st);
  else if (p.tn == 4) launch_tn<4>(a, p.waves_m, p.waves_n, p.tm, p.terms, p.lds_bytes, st);
  else launch_tn<5>(a, p.waves_m, p.waves_n, p.tm, p.terms, p.lds_bytes, st);
  return check_launch("conv_halo_bf16");
}

vcnn_status launch_conv_halo_bf16_prepared(const HaloBf16Plan& p, int n, int c, int h, int w, int m, int r, int s, int ph,
                                           int pw, const void* x, const void* wgt, int64_t w_so, int64_t w_si, int flip,
                                           const float* bias, void* y, int relu, void* x8_buf, void* wf_buf, hipStream_t st,
                                           float* y32, int accumulate) {
  if (x)
    if (vcnn_status e = relay_input(p, n, c, h, w, x, x8_buf, st)) return e;
  if (wgt)
    if (vcnn_status e = relay_kernels(p, c, m, r * s, wgt, w_so, w_si, flip, wf_buf, st)) return e;
  return launch_product(p, n, h, w, m, r, s, ph, pw, bias, y, relu, x8_buf, wf_buf, st, y32, accumulate);
}

// Three-term form (p planned with terms = 3): x_terms / w_terms hold the three bfloat16 terms of the float input and
// kernels, each term `x_term_bytes` / `w_term_bytes` after the one before; x8_bufs / wf_bufs take the three re-laid
// copies (3 x p.x8_bytes, 3 x p.wf_bytes).  One product kernel multiplies the six term pairs; the result is float.
vcnn_status launch_conv_halo_bf16_terms(const HaloBf16Plan& p, int n, int c, int h, int w, int m, int r, int s, int ph,
                                        int pw, const void* x_terms, size_t x_term_bytes, const void* w_terms,
                                        size_t w_term_bytes, int64_t w_so, int64_t w_si, const float* bias, float* y32,
                                        int relu, void* x8_bufs, void* wf_bufs, hipStream_t st) {
  for (int t = 0; t < 3; ++t) {
    if (vcnn_status e = relay_input(p, n, c, h, w, (const char*)x_terms + t * x_term_bytes, (char*)x8_bufs + t * p.x8_bytes, st))
      return e;
    if (vcnn_status e = relay_kernels(p, c, m, r * s, (const char*)w_terms + t * w_term_bytes, w_so, w_si, 0,
                                      (char*)wf_bufs + t * p.wf_bytes, st))
      return e;
  }
  return launch_product(p, n, h, w, m, r, s, ph, pw, bias, nullptr, relu, x8_bufs, wf_bufs, st, y32, 0);
}

// =========================================================================================================
// Filter gradient of the bf16 variant, dW[m][(c,r,s)] = sum_{n,pixel} dY[n][m][pixel] * xpad[n][c][pixel + (r,s)],
// as the mirror image of the kernel above: output maps on the MFMA rows, kernel-matrix columns (c,r,s) on
// the MFMA columns, contraction over (image, pixel).  The 8 contraction elements a lane feeds to one MFMA
// are the same pixel of 8 consecutive images, so both tensors are first re-laid image-interleaved:
//   x8n[n/8][c][h][w][8]                       staged (rows + halo) in LDS, read at tap_base(column) + pixel_offset(step);
//   dyf[n/8][row tile][run][step][lane][8]     dY in MFMA fragment order, read straight from L2.
// A chunk of the contraction is (image group, run of bh output rows); chunks are split over blockIdx.y and
// the partial products added in a fixed order by a second kernel.
// =========================================================================================================

// x8n[ng][pos][i8] = x[8 ng + i8][pos] (pos runs over c, h, w), zero for images >= N; x8n[total] = 0
__global__ __launch_bounds__(kThreads) void interleave_images_kernel(const bf16* __restrict__ x, uint4* __restrict__ x8n,
                                                                     int N, int64_t CHW, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i == 0) x8n[total] = make_uint4(0u, 0u, 0u, 0u);
  if (i >= total) return;
  const int64_t pos = i % CHW;
  const int ng = (int)(i / CHW);
  uint32_t v[8];
#pragma unroll
  for (int i8 = 0; i8 < 8; ++i8) {
    const int img = ng * 8 + i8;
    const bool ok = img < N;
    const uint16_t b = x[ok ? (int64_t)img * CHW + pos : 0].bits;
    v[i8] = ok ? b : 0u;
  }
  x8n[i] = make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
}

// dyf[ng][mt][run][jl][lane][i8] = dy[8 ng + i8][32 mt + lane % 32][run*bp + 2 jl + lane / 32] for pixels inside
// the run and the image, zero otherwise.  A thread owns one (map, pixel) and gathers its 8 images; consecutive
// lanes take consecutive pixels, so the reads are coalesced; the 16-byte writes of neighbouring maps fill
// whole cache lines between them.
__global__ __launch_bounds__(kThreads) void dy_fragments_kernel(const bf16* __restrict__ dy, uint4* __restrict__ dyf, int N,
                                                                int M, int P, int MT, int runs, int bp, int uch,
                                                                int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= total) return;
  const int u = (int)(i % uch);
  int64_t t = i / uch;
  const int run = (int)(t % runs);
  t /= runs;
  const int m = (int)(t % (MT * 32));
  const int ng = (int)(t / (MT * 32));
  const int p = run * bp + u;
  const bool inside = m < M && u < bp && p < P;
  uint32_t v[8];
#pragma unroll
  for (int i8 = 0; i8 < 8; ++i8) {
    const int img = ng * 8 + i8;
    const bool ok = inside && img < N;
    const uint16_t b = dy[ok ? ((int64_t)img * M + m) * P + p : 0].bits;
    v[i8] = ok ? b : 0u;
  }
  const int64_t frag = (((int64_t)ng * MT + m / 32) * runs + run) * (uch / 2) + u / 2;
  dyf[frag * 64 + (u & 1) * 32 + (m & 31)] =
      make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
}

// The same through LDS, for the launch: a block owns one image group, 32 maps, one run and 64 of its pixels.  It reads
// the 256 (image, map) rows of those pixels with consecutive lanes on consecutive pixels, and writes with consecutive
// lanes on consecutive maps - the order of a fragment - so that a wave's 16-byte stores fill 1 KB of contiguous memory
// (the kernel above stores 16 bytes per lane 1 KB apart and leaves it to the caches to assemble lines from blocks far
// apart in the grid: 0.040 ms for the 39 MB of cfg5 c3's dY).  Rows are padded to 66 elements: the lanes of a store,
// one map each, then read 32 different banks.
static constexpr int kFragPixels = 64, kFragPitch = 66;

__global__ __launch_bounds__(kThreads) void dy_fragments_tile_kernel(const bf16* __restrict__ dy, uint4* __restrict__ dyf,
                                                                     int N, int M, int P, int MT, int runs, int bp, int uch,
                                                                     int uchunks) {
  __shared__ uint16_t tile[8 * 32 * kFragPitch];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b = blockIdx.x;
  const int uc = b % uchunks;
  b /= uchunks;
  const int run = b % runs;
  b /= runs;
  const int mt = b % MT, ng = b / MT;
  const int u0 = uc * kFragPixels;
  {
    const int u = u0 + lane, p = run * bp + u;
    const bool pixel_ok = u < bp && p < P;
    // (two batches of 32 rows per wave: every load of a batch is in flight before the first is stored)
#pragma unroll 1
    for (int r0 = wave; r0 < 256; r0 += 128) {
      uint16_t v[32];
#pragma unroll
      for (int k = 0; k < 32; ++k) {  // row = (image in group, map in tile)
        const int row = r0 + 4 * k;
        const int img = ng * 8 + (row >> 5), m = mt * 32 + (row & 31);
        const bool ok = pixel_ok && img < N && m < M;
        const uint16_t t = dy[((int64_t)min(img, N - 1) * M + min(m, M - 1)) * P + (pixel_ok ? p : 0)].bits;
        v[k] = ok ? t : (uint16_t)0;
      }
#pragma unroll
      for (int k = 0; k < 32; ++k) tile[(r0 + 4 * k) * kFragPitch + lane] = v[k];
    }
  }
  __syncthreads();
  const int ml = tid & 31, ul = tid >> 5;
  const int64_t frag0 = (((int64_t)ng * MT + mt) * runs + run) * (uch / 2);
#pragma unroll
  for (int j = 0; j < kFragPixels / 8; ++j) {
    const int ulocal = ul + 8 * j, u = u0 + ulocal;
    if (u >= uch) break;
    uint32_t v[8];
#pragma unroll
    for (int i8 = 0; i8 < 8; ++i8) v[i8] = tile[(i8 * 32 + ml) * kFragPitch + ulocal];
    dyf[(frag0 + u / 2) * 64 + (u & 1) * 32 + ml] =
        make_uint4(v[0] | v[1] << 16, v[2] | v[3] << 16, v[4] | v[5] << 16, v[6] | v[7] << 16);
  }
}

struct FilterBf16Args {
  const uint4* x8n;   // [ng][c][h][w] positions of 8 images
  const uint4* zero;  // 16 zero bytes
  const uint4* dyf;   // [ng][mt][run][step][64 lanes] fragments
  int64_t x8n_term;   // TERMS > 1: distance between the terms of x8n, and of dyf, in 16-byte words
  int64_t dyf_term;
  float* out;         // [splits][m][K]
  int c, h, w, m, r, s, ph, pw, oh, ow;
  int K;              // c*r*s
  int tiles_m, mt_total;
  int runs, bh, bp;   // runs per image, output rows and pixels per run
  int uch, hpos, ccs, nr, wp;
  int nbuf;           // halo buffers: 2 = the next chunk is staged during the products of this one, 1 = between chunks
  int chunks, chunks_per_split;  // chunk = (image group, run)
};

// WAVES_N > 1: the waves of a block take different kernel-matrix columns of the same maps (they read the same dY
// fragments at about the same time, all but one from the first-level cache).  TERMS = 3: both operands as three
// bfloat16 terms each, the six largest term products per step - smallest first - into the same accumulators, with the
// operands of a step requested one step ahead, in order of first use, between the MFMAs (as in the forward kernel).
template <int WAVES_M, int WAVES_K, int TM, int TN, int WAVES_N = 1, int TERMS = 1>
__global__ __launch_bounds__(kThreads, 2) void filter_grad_bf16_kernel(FilterBf16Args a) {
  static_assert(WAVES_M * WAVES_K * WAVES_N * 64 == kThreads, "four waves per block");
  static_assert(TERMS == 1 || TERMS == 3, "plain bfloat16 operands, or floats as three terms");
  constexpr int PAIRS = TERMS == 1 ? 1 : 6;
  constexpr int kTermA[6] = {2, 0, 1, 1, 0, 0}, kTermB[6] = {0, 2, 1, 0, 1, 0};  // dY term, input term
  constexpr int BM = 32 * TM * WAVES_M, WN = 32 * TN, BN = WN * WAVES_N;
  extern __shared__ uint4 smem16[];
  int* const tbl = reinterpret_cast<int*>(smem16);  // [uch], per slab of 8 pixels: [half][4]
  uint4* const hbuf = smem16 + a.uch / 4;           // nbuf x TERMS x [ccs][nr][wp], each padded to hpos positions

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int wave_m = wave % WAVES_M, wave_k = (wave / WAVES_M) % WAVES_K, wave_n = wave / (WAVES_M * WAVES_K);
  const int tm = blockIdx.x % a.tiles_m;
  const int tk = blockIdx.x / a.tiles_m;
  const int i0 = tm * BM + wave_m * 32 * TM;  // first output map of this wave
  const int k0 = tk * BN;                     // first kernel-matrix column of the block
  const int kw0 = k0 + wave_n * WN;           // ... of this wave
  const int RS = a.r * a.s;
  const int plane = a.nr * a.wp;
  const int c_first = k0 / RS;

  // table: offset of pixel u of a run inside the halo tile; pixels beyond the run point at 0 (dY is zero there)
  for (int u = tid; u < a.uch; u += kThreads) {
    int off = 0;
    if (u < a.bp) {
      const int row = u / a.ow;
      off = row * a.wp + (u - row * a.ow);
    }
    const int sl = u >> 3, w8 = u & 7;
    tbl[sl * 8 + (w8 & 1) * 4 + (w8 >> 1)] = off;
  }

  int tap_base[TN];
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = min(kw0 + ni * 32 + l32, a.K - 1);
    const int c = col / RS;
    const int q = col - c * RS;
    const int r = q / a.s;
    tap_base[ni] = (c - c_first) * plane + r * a.wp + (q - r * a.s);
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int mi = 0; mi < TM; ++mi)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[mi][ni][q] = 0.f;

  const int id0 = blockIdx.y * a.chunks_per_split;
  const int id1 = min(a.chunks, id0 + a.chunks_per_split);
  const int steps = a.uch / 2;
  const int chunk_slabs = a.uch / 8;
  const int64_t mstride = (int64_t)a.runs * steps * 64;  // fragments per row tile of one image group
  auto frag_ptr = [&](int id, int sl) {
    const int ng = id / a.runs, run = id - ng * a.runs;
    return a.dyf + (((int64_t)ng * a.mt_total + i0 / 32) * a.runs + run) * steps * 64 + sl * 256 + lane;
  };

  // fragments on their way: a slab ahead (bfloat16 operands: a step is TM * TN MFMAs long) or a step ahead (three terms)
  constexpr int AHEAD = TERMS == 3 ? 1 : 4;
  uint4 af[TERMS][AHEAD][TM];
  const int first_sl = min(wave_k, chunk_slabs - 1);
  {
    const uint4* src = frag_ptr(id0, first_sl);
#pragma unroll
    for (int t = 0; t < TERMS; ++t)
#pragma unroll
      for (int i = 0; i < AHEAD; ++i)
#pragma unroll
        for (int mi = 0; mi < TM; ++mi) af[t][i][mi] = src[t * a.dyf_term + mi * mstride + i * 64];
  }

  const int dq = kThreads / a.wp, dr = kThreads - dq * a.wp;
  const int row_s = tid / a.wp, rx_s = tid - row_s * a.wp;
  const int cl_s = row_s / a.nr, ry_s = row_s - cl_s * a.nr;
  const int npos = a.ccs * plane;
  auto stage = [&](int id, uint4* dst) {
    const int ng = id / a.runs, run = id - ng * a.runs;
    const int ih0 = run * a.bh - a.ph;
    const uint4* xg = a.x8n + (int64_t)ng * a.c * a.h * a.w;
    int rx = rx_s, ry = ry_s, cl = cl_s;
    for (int b0 = wave * 64; b0 < npos; b0 += kThreads) {
      const int ih = ih0 + ry, iw = rx - a.pw, ch = c_first + cl;
      const bool ok = b0 + lane < npos && ch < a.c && ih >= 0 && ih < a.h && iw >= 0 && iw < a.w;
      const uint4* src = ok ? xg + (ch * a.h + ih) * a.w + iw : a.zero;
#pragma unroll
      for (int t = 0; t < TERMS; ++t) load_to_lds16(ok ? src + t * a.x8n_term : src, dst + t * a.hpos + b0);
      rx += dr;
      ry += dq;
      if (rx >= a.wp) rx -= a.wp, ++ry;
      while (ry >= a.nr) ry -= a.nr, ++cl;
    }
  };
  stage(id0, hbuf);

  for (int id = id0; id < id1; ++id) {
    const int run = id % a.runs;
    const int ulen = min(a.bh, a.oh - run * a.bh) * a.ow;  // valid pixels in this run
    const int slabs = (ulen + 7) >> 3;
    const uint4* halo = hbuf + ((id - id0) & (a.nbuf - 1)) * TERMS * a.hpos;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of the tile has landed
    __syncthreads();
    if (a.nbuf == 2 && id + 1 < id1) stage(id + 1, hbuf + ((id + 1 - id0) & 1) * TERMS * a.hpos);

    if constexpr (TERMS == 3) {
      auto read_offsets = [&](int sl, int (&dst)[4]) {
        const int4 o4 = *reinterpret_cast<const int4*>(tbl + sl * 8 + half * 4);
        dst[0] = o4.x, dst[1] = o4.y, dst[2] = o4.z, dst[3] = o4.w;
      };
      int o[4] = {0, 0, 0, 0};
      uint4 bfr[TERMS][TN];
      if (wave_k < slabs) {
        read_offsets(wave_k, o);
#pragma unroll
        for (int t = 0; t < TERMS; ++t)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni) bfr[t][ni] = halo[t * a.hpos + tap_base[ni] + o[0]];
      }
      for (int sl = wave_k; sl < slabs; sl += WAVES_K) {
        const int nsl = sl + WAVES_K;
        const uint4* csrc = frag_ptr(id, sl);
        const uint4* nsrc = nsl < slabs ? frag_ptr(id, nsl) : (id + 1 < id1 ? frag_ptr(id + 1, first_sl) : frag_ptr(id, sl));
        // offsets of this wave's next slab (past the chunk's last slab: any slab's - the words read with them are
        // dropped when the next chunk reads its own first step)
        int on[4];
        read_offsets(min(nsl, chunk_slabs - 1), on);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          uint4 cur[TERMS][TM], bnext[TERMS][TN];
          const uint4* nptr = i + 1 < 4 ? csrc + (i + 1) * 64 : nsrc;
          const int onext = i + 1 < 4 ? o[(i + 1) & 3] : on[0];
          constexpr int kOrderA[3] = {2, 0, 1}, kOrderB[3] = {0, 2, 1};  // the order of first use in the next step
#pragma unroll
          for (int k = 0; k < TERMS; ++k)
#pragma unroll
            for (int mi = 0; mi < TM; ++mi) {
              const int t = kOrderA[k];
              cur[t][mi] = af[t][0][mi];
              af[t][0][mi] = nptr[t * a.dyf_term + mi * mstride];
            }
#pragma unroll
          for (int k = 0; k < TERMS; ++k)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
              const int t = kOrderB[k];
              bnext[t][ni] = halo[t * a.hpos + tap_base[ni] + onext];
            }
#pragma unroll
          for (int pr = 0; pr < PAIRS; ++pr)
#pragma unroll
            for (int mi = 0; mi < TM; ++mi)
#pragma unroll
              for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(cur[kTermA[pr]][mi], bfr[kTermB[pr]][ni], acc[mi][ni]);
          // issue order: one fragment load and one halo read after every TM * TN MFMAs, in the shadow of the matrix pipe
#pragma unroll
          for (int k = 0; k < TERMS * TM; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x008, PAIRS * TN / TERMS, 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                   // global read
            if (k < TERMS * TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
          }
#pragma unroll
          for (int t = 0; t < TERMS; ++t)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) bfr[t][ni] = bnext[t][ni];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = on[i];
      }
    } else {
      for (int sl = wave_k; sl < slabs; sl += WAVES_K) {
        const int nsl = sl + WAVES_K;
        const uint4* nsrc = nsl < slabs ? frag_ptr(id, nsl) : (id + 1 < id1 ? frag_ptr(id + 1, first_sl) : frag_ptr(id, sl));
        const int4 o4 = *reinterpret_cast<const int4*>(tbl + sl * 8 + half * 4);
        const int o[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          uint4 bfr[TN], cur[TM];
#pragma unroll
          for (int ni = 0; ni < TN; ++ni) bfr[ni] = halo[tap_base[ni] + o[i]];
#pragma unroll
          for (int mi = 0; mi < TM; ++mi) {
            cur[mi] = af[0][i][mi];
            af[0][i][mi] = nsrc[mi * mstride + i * 64];
          }
          // keep the fragment loads of the next slab ahead of this step's MFMAs: a full slab of lead time
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) acc[mi][ni] = mfma_bf16(cur[mi], bfr[ni], acc[mi][ni]);
        }
      }
    }
    if (a.nbuf == 1 && id + 1 < id1) {  // one buffer: every wave is done reading it, then it is refilled
      __syncthreads();
      stage(id + 1, hbuf);
    }
  }

  if (WAVES_K > 1) {  // contraction split between waves: add the partial sums in wave order through LDS
    float* red = reinterpret_cast<float*>(smem16);  // [TM*TN*16][64 lanes]
#pragma unroll 1
    for (int k = 1; k < WAVES_K; ++k) {
      __syncthreads();
      if (wave_k == k) {
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int q = 0; q < 16; ++q) red[(((wave_m * TM + mi) * TN + ni) * 16 + q) * 64 + lane] = acc[mi][ni][q];
      }
      __syncthreads();
      if (wave_k == 0) {
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
          for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[mi][ni][q] += red[(((wave_m * TM + mi) * TN + ni) * 16 + q) * 64 + lane];
      }
    }
    if (wave_k != 0) return;
  }

  float* dst = a.out + (int64_t)blockIdx.y * a.m * a.K;
#pragma unroll
  for (int ni = 0; ni < TN; ++ni) {
    const int col = kw0 + ni * 32 + l32;
    if (col >= a.K) continue;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int m = i0 + mi * 32 + 8 * (q >> 2) + 4 * half + (q & 3);
        if (m < a.m) dst[(int64_t)m * a.K + col] = acc[mi][ni][q];
      }
  }
}

// A 1x1 unpadded layer does not care how its pixels are arranged: seen as a P x 1 image, a "run of rows" is
// any run of pixels, which keeps the LDS tile (channels x run) small however wide the image is.
static ConvGeom flatten_pointwise(const ConvGeom& g) {
  ConvGeom f = g;
  if (g.r == 1 && g.s == 1 && g.ph == 0 && g.pw == 0 && g.P <= 0x7fffffffLL) {
    f.h = f.oh = (int)g.P;
    f.w = f.ow = 1;
  }
  return f;
}

bool filter_grad_bf16_plan(const ConvGeom& g0, FilterGradBf16Plan* p, int terms) {
  const ConvGeom g = flatten_pointwise(g0);
  const int rs = g.r * g.s;
  if ((int64_t)g.c * g.h * g.w > 0x7fffffffLL || g.K > 0x7fffffffLL) return false;
  p->terms = terms, p->waves_n = 1;
  int tn = 0;
  if (terms == 3) {
    // built for many maps: the four waves take 64 columns each of the same 64 maps (the registers of three terms
    // leave room for the accumulators of 64 x 64 wave tiles)
    if (g.M <= 128) return false;
    p->waves_m = 1, p->waves_n = 4, p->tm = 2, tn = 2;
  } else {
    p->waves_m = g.M > 128 ? 4 : (g.M > 64 ? 2 : 1);
    p->tm = g.M <= 32 ? 1 : 2;
    // column tile: least padding of the kernel-matrix width, wider on ties
    int64_t padded = 0;
    for (int t : kTnChoices) {
      const int64_t pd = ceil_div(g.K, 32 * t) * 32 * t;
      if (tn == 0 || pd <= padded) tn = t, padded = pd;
    }
  }
  const int waves_k = 4 / (p->waves_m * p->waves_n);
  const int bm = 32 * p->tm * p->waves_m;
  const int tiles_m = (int)ceil_div(g.M, bm);
  const int bn = 32 * tn * p->waves_n;
  p->tn = tn;
  p->wp = g.w + 2 * g.pw;
  // channels a run of bn columns can touch (one when the column tiles never straddle a channel)
  p->ccs = rs % bn == 0 ? 1 : (int)std::min<int64_t>(g.c, (bn + rs - 2) / rs + 1);
  const size_t red_bytes = waves_k > 1 ? (size_t)p->waves_m * p->tm * tn * 16 * 64 * sizeof(float) : 0;
  if (red_bytes > kLdsBudget) return false;
  // most output rows per run whose halo tile fits twice - or, three planes of a large kernel, once: then a chunk is
  // staged between the products of two chunks, not during them, and the other resident block covers the gap
  int bh = 0;
  for (p->nbuf = 2; p->nbuf >= (terms == 3 ? 1 : 2) && bh == 0; --p->nbuf) {
    for (int t = 1; t <= g.oh; ++t) {
      const int uch = (int)ceil_div((int64_t)t * g.ow, 8) * 8;
      const size_t hpos = ((size_t)p->ccs * (t + g.r - 1) * p->wp + 63) & ~(size_t)63;
      if ((size_t)uch * 4 + p->nbuf * terms * hpos * 16 > kLdsBudget || uch > 4096) break;
      bh = t;
    }
    if (bh) break;
  }
  if (bh == 0) return false;
  p->bh = bh, p->bp = bh * g.ow, p->nr = bh + g.r - 1;
  p->uch = (int)ceil_div((int64_t)p->bp, 8) * 8;
  p->hpos = (int)(((size_t)p->ccs * p->nr * p->wp + 63) & ~(size_t)63);
  p->lds_bytes = std::max((size_t)p->uch * 4 + p->nbuf * terms * (size_t)p->hpos * 16, red_bytes);
  p->runs = (int)ceil_div(g.oh, bh);
  p->ngroups = (g.n + 7) / 8;
  p->chunks = p->ngroups * p->runs;
  const int64_t tiles = (int64_t)tiles_m * ceil_div(g.K, bn);
  int64_t want = ceil_div(512, tiles);
  if (terms == 3) {
    // long blocks that keep the matrix pipe busy: the 256 CUs share them evenly when there are many per CU, or a
    // whole number; of the even splits of the chunks, the first that leaves the last CU at least 90 % of a share
    for (int64_t wn = want; wn <= p->chunks; ++wn) {
      if (p->chunks % wn) continue;
      const double per_cu = (double)tiles * wn / 256.0;
      if (per_cu / std::ceil(per_cu) >= 0.9) {
        want = wn;
        break;
      }
    }
  }
  if (want > p->chunks) want = p->chunks;
  if (want < 1) want = 1;
  p->chunks_per_split = (int)ceil_div(p->chunks, want);
  p->splits = (int)ceil_div(p->chunks, p->chunks_per_split);
  p->mt_total = tiles_m * (bm / 32);
  p->x8n_bytes = (((size_t)p->ngroups * g.c * g.h * g.w + 1) * 16 + 255) & ~(size_t)255;
  p->dyf_bytes = ((size_t)p->ngroups * p->mt_total * p->runs * (p->uch / 2) * 64 * 16 + 255) & ~(size_t)255;
  p->partial_bytes = p->splits > 1 ? (size_t)p->splits * g.M * g.K * sizeof(float) : 0;
  return tiles <= 0x7fffffffLL && p->splits <= 65535;
}

template <int WAVES_M, int WAVES_K, int TM, int TN, int WAVES_N = 1, int TERMS = 1>
static void launch_filter_one(const FilterBf16Args& a, unsigned tiles, unsigned splits, size_t lds, hipStream_t st) {
  auto kernel = filter_grad_bf16_kernel<WAVES_M, WAVES_K, TM, TN, WAVES_N, TERMS>;
  static bool opted = false;
  if (!opted) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kLdsBudget);
    opted = true;
  }
  hipLaunchKernelGGL(kernel, dim3(tiles, splits), dim3(kThreads), lds, st, a);
}

template <int TN>
static void launch_filter_tn(const FilterBf16Args& a, int waves_m, int tm, unsigned tiles, unsigned splits, size_t lds,
                             hipStream_t st) {
  if (waves_m == 4) launch_filter_one<4, 1, 2, TN>(a, tiles, splits, lds, st);
  else if (waves_m == 2) launch_filter_one<2, 2, 2, TN>(a, tiles, splits, lds, st);
  else if (tm == 2) launch_filter_one<1, 4, 2, TN>(a, tiles, splits, lds, st);
  else launch_filter_one<1, 4, 1, TN>(a, tiles, splits, lds, st);
}

vcnn_status launch_filter_grad_bf16(const FilterGradBf16Plan& p, const ConvGeom& g0, const void* x, const void* dy,
                                    float* dw, void* workspace, hipStream_t st, int accumulate) {
  return launch_filter_grad_bf16_prepared(p, g0, x, dy, dw, workspace, (char*)workspace + p.x8n_bytes,
                                          (float*)((char*)workspace + p.x8n_bytes + p.dyf_bytes), st, accumulate);
}

static vcnn_status relay_images(const FilterGradBf16Plan& p, const ConvGeom& g, const void* x, void* x8n_buf, hipStream_t st) {
  const int64_t chw = (int64_t)g.c * g.h * g.w;
  const int64_t total = (int64_t)p.ngroups * chw;
  hipLaunchKernelGGL(interleave_images_kernel, dim3((unsigned)ceil_div(total, kThreads)), dim3(kThreads), 0, st,
                     (const bf16*)x, (uint4*)x8n_buf, g.n, chw, total);
  return check_launch("interleave_images");
}

static vcnn_status relay_dy(const FilterGradBf16Plan& p, const ConvGeom& g, const void* dy, void* dyf_buf, hipStream_t st) {
  const int uchunks = (int)ceil_div(p.uch, kFragPixels);
  const int64_t blocks = (int64_t)p.ngroups * p.mt_total * p.runs * uchunks;
  if (blocks <= 0x7fffffffLL && p.uch >= kFragPixels / 2) {  // (short runs would leave most of a block's pixels empty)
    hipLaunchKernelGGL(dy_fragments_tile_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, (const bf16*)dy,
                       (uint4*)dyf_buf, g.n, (int)g.M, (int)g.P, p.mt_total, p.runs, p.bp, p.uch, uchunks);
    return check_launch("dy_fragments_tile");
  }
  const int64_t total = (int64_t)p.ngroups * p.mt_total * 32 * p.runs * p.uch;
  hipLaunchKernelGGL(dy_fragments_kernel, dim3((unsigned)ceil_div(total, kThreads)), dim3(kThreads), 0, st,
                     (const bf16*)dy, (uint4*)dyf_buf, g.n, (int)g.M, (int)g.P, p.mt_total, p.runs, p.bp, p.uch, total);
  return check_launch("dy_fragments");
}

// the product on re-laid operands (g flattened), slices summed into dw (added to its contents when `accumulate`)
static vcnn_status launch_filter_product(const FilterGradBf16Plan& p, const ConvGeom& g, float* dw, const void* x8n_buf,
                                         const void* dyf_buf, float* partial, hipStream_t st, int accumulate) {
  const uint4* x8n = (const uint4*)x8n_buf;
  const int64_t chw = (int64_t)g.c * g.h * g.w;
  FilterBf16Args a{};
  // accumulate: dw += the product (the slice sum takes dw as its addend); the workspace then holds at least one slice
  a.x8n = x8n, a.zero = x8n + (int64_t)p.ngroups * chw, a.dyf = (const uint4*)dyf_buf;
  a.x8n_term = (int64_t)(p.x8n_bytes / 16), a.dyf_term = (int64_t)(p.dyf_bytes / 16);  // (read by the three-term form only)
  a.out = (p.splits > 1 || accumulate) ? partial : dw;
  a.c = g.c, a.h = g.h, a.w = g.w, a.m = g.k, a.r = g.r, a.s = g.s, a.ph = g.ph, a.pw = g.pw, a.oh = g.oh, a.ow = g.ow;
  a.K = (int)g.K;
  a.tiles_m = (int)ceil_div(g.M, 32 * p.tm * p.waves_m), a.mt_total = p.mt_total;
  a.runs = p.runs, a.bh = p.bh, a.bp = p.bp;
  a.uch = p.uch, a.hpos = p.hpos, a.ccs = p.ccs, a.nr = p.nr, a.wp = p.wp, a.nbuf = p.nbuf;
  a.chunks = p.chunks, a.chunks_per_split = p.chunks_per_split;
  const unsigned tiles = (unsigned)(a.tiles_m * ceil_div(g.K, 32 * p.tn * p.waves_n));
  if (p.terms == 3) launch_filter_one<1, 1, 2, 2, 4, 3>(a, tiles, (unsigned)p.splits, p.lds_bytes, st);
  else if (p.tn == 2) launch_filter_tn<2>(a, p.waves_m, p.tm, tiles, (unsigned)p.splits, p.lds_bytes, st);
  else if (p.tn == 4) launch_filter_tn<4>(a, p.waves_m, p.tm, tiles, (unsigned)p.splits, p.lds_bytes, st);
  else launch_filter_tn<5>(a, p.waves_m, p.tm, tiles, (unsigned)p.splits, p.lds_bytes, st);
  if (vcnn_status e = check_launch("filter_grad_bf16")) return e;
  if (p.splits == 1 && !accumulate) return VCNN_OK;
  if (accumulate)  // "bias" of element i = dw[i]
    return launch_sum_slices(partial, dw, dw, VCNN_F32, g.M * g.K, p.splits, 1, (int)(g.M * g.K), 0, st);
  return launch_sum_slices(partial, nullptr, dw, VCNN_F32, g.M * g.K, p.splits, 1, 1, 0, st);
}

vcnn_status launch_filter_grad_bf16_prepared(const FilterGradBf16Plan& p, const ConvGeom& g0, const void* x, const void* dy,
                                             float* dw, void* x8n_buf, void* dyf_buf, float* partial, hipStream_t st,
                                             int accumulate) {
  const ConvGeom g = flatten_pointwise(g0);
  if (x)
    if (vcnn_status e = relay_images(p, g, x, x8n_buf, st)) return e;
  if (dy)
    if (vcnn_status e = relay_dy(p, g, dy, dyf_buf, st)) return e;
  return launch_filter_product(p, g, dw, x8n_buf, dyf_buf, partial, st, accumulate);
}

// Three-term form (p planned with terms = 3): x_terms / dy_terms hold the three bfloat16 terms of the float input and
// output gradient, each term `x_term_bytes` / `dy_term_bytes` after the one before; x8n_bufs / dyf_bufs take the three
// re-laid copies (3 x p.x8n_bytes, 3 x p.dyf_bytes), `partial` the slices.  One product kernel multiplies the six pairs.
vcnn_status launch_filter_grad_bf16_terms(const FilterGradBf16Plan& p, const ConvGeom& g0, const void* x_terms,
                                          size_t x_term_bytes, const void* dy_terms, size_t dy_term_bytes, float* dw,
                                          void* x8n_bufs, void* dyf_bufs, float* partial, hipStream_t st) {
  const ConvGeom g = flatten_pointwise(g0);
  for (int t = 0; t < 3; ++t) {
    if (vcnn_status e = relay_images(p, g, (const char*)x_terms + t * x_term_bytes, (char*)x8n_bufs + t * p.x8n_bytes, st)) return e;
    if (vcnn_status e = relay_dy(p, g, (const char*)dy_terms + t * dy_term_bytes, (char*)dyf_bufs + t * p.dyf_bytes, st)) return e;
  }
  return launch_filter_product(p, g, dw, x8n_bufs, dyf_bufs, partial, st, 0);
}

}  // namespace vcnn
