// Strided convolution (Section 3, listing sconv2d) on the int8 matrix core, for a multiple of 32 filters and a
// reduction C * KH * KW that is a multiple of 4 (any filter size and strides):
//
//   O(n,f,h,w) = B(f) + sum_{c,kh,kw} I(n,c, sh*h + kh, sw*w + kw) * W(f,c,kh,kw)
//
// As a contraction this is the transposed matmul of gemm_i8.hpp: the rows of "X" are the filters (their
// C * KH * KW taps are contiguous in W), the rows of "Y" are the N * OH * OW output pixels of the whole batch, whose
// taps are gathered from I, and the reduction runs over the taps in W's order.  The arithmetic is that kernel's: in
// every block of 128 taps each filter and each pixel is scaled so that its largest magnitude maps to 0x7F7F7F7E,
// rounded to a 32-bit integer and cut into four signed 8-bit digits; the digit products with k + l >= MIND are
// summed exactly in int32 (v_mfma_i32_16x16x64_i8), scaled back and added over the blocks in fp64; one rounding to
// fp32.  The last block of a reduction that is not a multiple of 128 is filled with zeros.
//
// One workgroup of 8 wavefronts = TF filters against 16 * NT consecutive pixels: TF = 128 with NT = 1 .. 4, or, where
// the number of filters is a multiple of 64 (of 32) only, TF = 64 with NT = 2, 4, 6, 8 (TF = 32 with NT = 4, 8, 12;
// the first four wavefronts stage the filters); the host picks NT so that one round of workgroups covers the image
// batch where it can.
// Staging: the filter half is gemm_i8.hpp's X half (a thread owns 32 taps of one filter, row maximum across its
// quad; with 64 filters 16 taps -- one MFMA step of a chunk -- and the maximum across 8 lanes).  The pixel half: a
// thread owns one group of 4 consecutive taps of the block (group g = tid / 16: 32 groups) for NT pixels
// (16 i + tid % 16), so a load instruction of a wavefront covers 16 consecutive pixels for each of 4 groups; the byte
// offsets of the block's taps relative to a pixel's first input element come from a table in LDS (built once per
// workgroup: one division per tap there instead of one per gathered element).  A pixel's 128 taps are
// spread over 32 threads in all 8 wavefronts, so its maximum is formed by LDS atomics (ds_max_u32) one block ahead:
// the gathers of block t + 1 are issued before block t is contracted, their maxima are posted after it, and the
// barrier that ends block t publishes them.
// Contraction: wavefront w holds the operands of filter tile w % (TF / 16) in registers and runs them against its
// pixel tiles (all NT of them at 128 filters; at 64 (32) filters the tiles i with i % 2 = w / 4 (i % 4 = w / 2));
// MFMA rows = pixels, columns = filters, so a lane ends up with 4 consecutive pixels of one filter.
//
// Groups (the grouped convolution of Section 7 with stride 1): blockIdx.z is the group; a group's channels, filters
// and outputs are contiguous slices of I, Wt, bias and O, so only base offsets change.
//
// A filter or a pixel whose taps hold Inf or NaN gives NaN in every output of that filter (pixel).
#pragma once
#include "gemm_i8.hpp"

namespace tc355 {

struct SconvI8Args {
  const float* I;     // [N][C][H][W] (G = 1), fewer than 2^30 elements
  const float* Wt;    // [F][C][KH][KW]
  const float* bias;  // [F] or nullptr
  float* O;           // [N][F][OH][OW]
  int C, F, H, W, KH, KW, sh, sw, OH, OW;
  int G;              // groups (blockIdx.z): I is [N][G][C][H][W], Wt [G][F][C][KH][KW], bias [G * F], O [N][G][F][OH][OW]
  int K;              // C * KH * KW
  int P;              // N * OH * OW
};

constexpr int SI8_KB = 128, SI8_THREADS = 512, SI8_WAVES = SI8_THREADS / WAVE;
constexpr int SI8_STEPS = SI8_KB / 64;
constexpr int SI8_RS = SI8_KB + 32;  // row stride of a digit plane: see GI8_RS
// pixel tiles per wavefront: five and six do not fit the 256 registers of a wavefront
constexpr int SI8_MAX_TILES_PER_WAVE = 4;

template <int TF, int NT>
struct SconvI8Geom {
  static_assert(TF == 128 || TF == 64 || TF == 32, "8, 4 or 2 filter tiles");
  static constexpr int FT = TF / 16;                 // filter tiles
  static constexpr int PG = SI8_WAVES / FT;          // groups of wavefronts that share the pixel tiles out: 1, 2 or 4
  static constexpr int NTW = NT / PG;                // pixel tiles per wavefront
  static_assert(NT % PG == 0 && NTW >= 1 && NTW <= SI8_MAX_TILES_PER_WAVE, "16 to 64 pixels per wavefront");
  static constexpr int TPR = TF == 128 ? 4 : 8;      // threads that stage one filter's block
  static constexpr int XS = 4 * SI8_STEPS / TPR;     // MFMA steps of the block that one of them stages: 2 or 1
  static constexpr int XTHREADS = TF * TPR;          // threads with a share of the filters: all, or (32 filters) the first 256
  static constexpr int TP = 16 * NT;                 // pixels per workgroup
  static constexpr int ROWS = TF + TP;               // rows staged per block: filters, then pixels
  static constexpr int PLANE = ROWS * SI8_RS;
  static constexpr int INVS = 4 * PLANE;             // ROWS inverse scales (fp64)
  static constexpr int RMAX = INVS + ROWS * 8;       // [2][TP] largest magnitudes of the pixels' blocks
  static constexpr int TABLE = RMAX + 2 * TP * 4;    // [blocks * 128] byte offsets of the taps, 0 past the end
  static constexpr int64_t lds_bytes(int64_t blocks) { return TABLE + blocks * SI8_KB * 4; }
  static_assert(INVS % 16 == 0 && RMAX % 16 == 0 && TABLE % 16 == 0, "16-byte LDS accesses");
};

template <int TF, int NT, int MIND>
__global__ __launch_bounds__(SI8_THREADS, 1) void sconv_i8_kernel(SconvI8Args p) {
  static_assert(MIND == 2 || MIND == 3, "13 or 10 digit products");
  using Gm = SconvI8Geom<TF, NT>;
  constexpr int TP = Gm::TP, PLANE = Gm::PLANE, FT = Gm::FT, PG = Gm::PG, NTW = Gm::NTW, TPR = Gm::TPR, XS = Gm::XS;
  constexpr bool XALL = Gm::XTHREADS == SI8_THREADS;
  extern __shared__ __attribute__((aligned(16))) char si8_lds[];
  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int K = p.K, nb = (K + SI8_KB - 1) / SI8_KB;
  const int f0 = blockIdx.y * TF;
  const int p0 = blockIdx.x * TP;
  const int OHW = p.OH * p.OW;
  const int G = p.G, grp = blockIdx.z;
  double* invs = reinterpret_cast<double*>(si8_lds + Gm::INVS);
  unsigned* rmax = reinterpret_cast<unsigned*>(si8_lds + Gm::RMAX);
  unsigned* table = reinterpret_cast<unsigned*>(si8_lds + Gm::TABLE);

  // ---- the taps' byte offsets from a pixel's first input element, in W's order (c, kh, kw)
  {
    const int HW = p.H * p.W, KW = p.KW, KHW = p.KH * p.KW;
    for (int k = tid; k < nb * SI8_KB; k += SI8_THREADS) {
      const int c = k / KHW, t = k - c * KHW, kh = t / KW, kw = t - kh * KW;
      table[k] = k < K ? 4u * (unsigned)(c * HW + kh * p.W + kw) : 0u;  // past the end: any element of I; the value is dropped
    }
    if (tid < 2 * TP) rmax[tid] = 0u;
  }

  // ---- staging role, filters: 16 slots per MFMA step of filter tid / TPR (chunk cx of the step); slot 16 c + 4 j + e
  // of step s holds tap 64 s + 16 j + 4 c + e of the block.  With 128 filters a thread stages both steps, with 64
  // the step xs0 only.
  const int xrow = tid / TPR, cx = tid & 3, xs0 = XS == 2 ? 0 : (tid >> 2) & 1;
  const bool xon = XALL || wave < Gm::XTHREADS / WAVE;  // (whole wavefronts: uniform)
  const float* xsrc = p.Wt + ((int64_t)grp * p.F + f0 + xrow) * K + 4 * cx;
  f4 rx[XS][4];
  // ---- staging role, pixels: taps 64 s + 16 j + 4 c .. + 3 of the block (group g = (s, j, c)) of pixels 16 i + pl
  const int g = tid >> 4, pl = tid & 15;
  const int kg = 64 * (g >> 4) + 16 * ((g >> 2) & 3) + 4 * (g & 3);              // first tap of the group in its block
  const int ycol = 16 * (4 * (g >> 4) + (g & 3)) + 4 * ((g >> 2) & 3);           // its 4 bytes in a digit-plane row
  unsigned ybase[NT];  // byte offset of the pixel's first input element
#pragma unroll
  for (int i = 0; i < NT; i++) {
    const int pi = min(p0 + 16 * i + pl, p.P - 1);  // pixels past the end repeat the last one (never stored)
    const int img = pi / OHW, rem = pi - img * OHW, oh = rem / p.OW, ow = rem - oh * p.OW;
    ybase[i] = 4u * (unsigned)(((img * G + grp) * p.C * p.H + oh * p.sh) * p.W + ow * p.sw);
  }
  f4 ry[NT];

  auto fetch_x = [&](int blk, int u) {  // this thread's u-th step (64 taps) of the block
    if (!xon) return;
    const int st = xs0 + u;
    const float* xs = xsrc + blk * SI8_KB + 64 * st;
    if (blk * SI8_KB + SI8_KB <= K) {
#pragma unroll
      for (int j = 0; j < 4; j++) rx[u][j] = *reinterpret_cast<const f4*>(xs + 16 * j);
    } else {
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const bool in = blk * SI8_KB + 64 * st + 16 * j + 4 * cx < K;  // K is a multiple of 4: whole pieces
        rx[u][j] = in ? *reinterpret_cast<const f4*>(xs + 16 * j) : f4{0.f, 0.f, 0.f, 0.f};
      }
    }
  };
  auto fetch_y = [&](int blk) {
    const i4 off = *reinterpret_cast<const i4*>(table + blk * SI8_KB + kg);
    const char* src = reinterpret_cast<const char*>(p.I);
#pragma unroll
    for (int i = 0; i < NT; i++)
#pragma unroll
      for (int e = 0; e < 4; e++) ry[i][e] = *reinterpret_cast<const float*>(src + (ybase[i] + (unsigned)off[e]));
  };
  // largest magnitudes of the fetched pixel taps, posted for the block that is staged next (buffer `buf`)
  auto post_max = [&](int buf, int blk) {
    if (blk * SI8_KB + SI8_KB > K) {  // the end of the reduction: taps past it count as zeros
#pragma unroll
      for (int i = 0; i < NT; i++)
#pragma unroll
        for (int e = 0; e < 4; e++) ry[i][e] = blk * SI8_KB + kg + e < K ? ry[i][e] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < NT; i++) {
      int sm = 0;
      unsigned um = 0;
      gi8_absmax4(ry[i], sm, um);
      __hip_atomic_fetch_max(&rmax[buf * TP + 16 * i + pl], (unsigned)gi8_magnitude(sm, um), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  };
  double xscale;  // of this thread's filter in the block being staged
  auto scale_x = [&]() {  // filters: row shared by TPR neighbouring lanes
    if (!xon) return;
    int sm = 0;
    unsigned um = 0;
#pragma unroll
    for (int u = 0; u < XS; u++)
#pragma unroll
      for (int j = 0; j < 4; j++) gi8_absmax4(rx[u][j], sm, um);
    int v = gi8_magnitude(sm, um);
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
    if constexpr (TPR == 8) v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));  // row_half_mirror: the other quad
    double inverse;
    gi8_scales((unsigned)v, xscale, inverse);
    invs[xrow] = inverse;  // the lanes of the row write the same value
  };
  auto slice_x = [&](int u) {  // 16 elements of this thread's u-th step
    if (!xon) return;
    int y[4][4];
#pragma unroll
    for (int j = 0; j < 4; j++) gi8_digits4(rx[u][j], xscale, y[j]);
    char* dst = si8_lds + xrow * SI8_RS + 16 * (4 * (xs0 + u) + cx);
#pragma unroll
    for (int k = 0; k < 4; k++) {
      i4 rec;
      rec.x = y[0][k]; rec.y = y[1][k]; rec.z = y[2][k]; rec.w = y[3][k];
      *reinterpret_cast<i4*>(dst + k * PLANE) = rec;
    }
  };
  auto slice_y = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NT; i++) {  // pixels: 4 elements, row shared by 32 threads
      const int row = 16 * i + pl;
      double scale, inverse;
      gi8_scales(rmax[buf * TP + row], scale, inverse);
      int y[4];
      gi8_digits4(ry[i], scale, y);
      char* dst = si8_lds + (TF + row) * SI8_RS + ycol;
#pragma unroll
      for (int k = 0; k < 4; k++) *reinterpret_cast<int*>(dst + k * PLANE) = y[k];
      if (g == 0) invs[TF + row] = inverse * 16777216.0;  // 2^24: the weight of the lowest kept diagonal
    }
    if (tid < TP) rmax[(buf ^ 1) * TP + tid] = 0u;  // last read one block ago; next written after the coming barrier
  };

  // ---- contraction role: filter tile ft against the pixel tiles pg, pg + PG, ..
  const int ft = wave % FT, pg = wave / FT;
  double acc[NTW][4];
#pragma unroll
  for (int i = 0; i < NTW; i++)
#pragma unroll
    for (int v = 0; v < 4; v++) acc[i][v] = 0.0;
  // one_step: the block holds at most 64 taps (the end of a reduction), its second MFMA step would multiply zeros
  auto contract = [&](bool one_step) {
    i4 xa[SI8_STEPS][4];
#pragma unroll
    for (int s = 0; s < SI8_STEPS; s++) {
      const char* xb = si8_lds + (16 * ft + r16) * SI8_RS + 16 * (4 * s + q);
#pragma unroll
      for (int l = 0; l < 4; l++) xa[s][l] = *reinterpret_cast<const i4*>(xb + l * PLANE);
    }
    const double fx = invs[16 * ft + r16];
    // order: no two consecutive products on one diagonal
    constexpr int ND = 7 - MIND, NP = MIND == 3 ? 10 : 13;
    constexpr int PK[13] = {3, 2, 3, 3, 2, 1, 2, 1, 0, 3, 2, 1, 0};  // the last three: the diagonal k + l = 2
    constexpr int PL[13] = {0, 1, 1, 2, 2, 2, 3, 3, 3, 3, 0, 1, 2};
    i4 d[ND];  // d[i]: diagonal k + l = MIND + i
    auto mma = [&](int i, i4 (&dd)[ND]) {
#pragma unroll
      for (int s = 0; s < SI8_STEPS; s++) {
        if (s == 1 && one_step) break;
        const char* yb = si8_lds + (TF + 16 * (pg + PG * i) + r16) * SI8_RS + 16 * (4 * s + q);
        i4 ya[4];
#pragma unroll
        for (int k = 0; k < 4; k++) ya[k] = *reinterpret_cast<const i4*>(yb + k * PLANE);
        bool begun[ND] = {};  // (compile-time after unrolling) the first product of a diagonal starts from a literal zero
#pragma unroll
        for (int pr = 0; pr < NP; pr++) {
          const int dg = PK[pr] + PL[pr] - MIND;
          dd[dg] = mfma_i8(ya[PK[pr]], xa[s][PL[pr]], s == 0 && !begun[dg] ? i4{0, 0, 0, 0} : dd[dg]);
          begun[dg] = true;
        }
      }
    };
    auto epilogue = [&](int i, const i4 (&dd)[ND]) {
#pragma unroll
      for (int v = 0; v < 4; v++) {
        // 128 terms of at most 2^14 per digit pair: 2^21 x 256 + 2 x 2^21 and 3 x 2^21 x 256 + 4 x 2^21, below 2^31
        const int hi = dd[ND - 1][v] * 256 + dd[ND - 2][v], lo = dd[ND - 3][v] * 256 + dd[ND - 4][v];
        double rr = __builtin_fma((double)hi, 65536.0, (double)lo);
        if constexpr (MIND == 2) rr = __builtin_fma((double)dd[0][v], 0.00390625, rr);
        acc[i][v] = __builtin_fma(rr, invs[TF + 16 * (pg + PG * i) + 4 * q + v] * fx, acc[i][v]);
      }
    };
#pragma unroll
    for (int i = 0; i < NTW; i++) {
      __builtin_amdgcn_sched_barrier(0);  // one tile's operands at a time: hoisted reads of all tiles do not fit the registers
      mma(i, d);
      epilogue(i, d);
    }
  };

  __syncthreads();  // the table
#pragma unroll
  for (int u = 0; u < XS; u++) fetch_x(0, u);
  fetch_y(0);
  post_max(0, 0);
  __syncthreads();
  for (int t = 0; t < nb; t++) {
    // the next block's loads as soon as this block's registers are free: the gathers' address work (8 clocks per
    // instruction and compute unit) runs under the filters' slicing
    slice_y(t & 1);
    __builtin_amdgcn_sched_barrier(0);
    if (t + 1 < nb) fetch_y(t + 1);
    scale_x();
#pragma unroll
    for (int u = 0; u < XS; u++) slice_x(u);
    __builtin_amdgcn_sched_barrier(0);
    if (t + 1 < nb) {  // (a step's loads right after that step's slicing measured 1-2 % slower)
#pragma unroll
      for (int u = 0; u < XS; u++) fetch_x(t + 1, u);
    }
    __syncthreads();
    contract(K - t * SI8_KB <= 64);
    if (t + 1 < nb) post_max((t + 1) & 1, t + 1);
    __syncthreads();
  }

  // ---- outputs: staged in the digit planes' LDS (free now) as [filter][pixel], then written as runs of consecutive
  // pixels of one filter (a lane's own 4 pixels of 16 filters per instruction would be 64 separate 4-byte writes)
  constexpr int OS = TP + 1;  // row stride in floats: odd, so the 16 filters of a wavefront's write fall into 16 banks
  float* ostage = reinterpret_cast<float*>(si8_lds);
  int* pxoff = reinterpret_cast<int*>(si8_lds + TF * OS * 4);  // [TP] offset of (image, pixel) in O for filter 0, -1 past the end
  static_assert(TF * OS * 4 + TP * 4 <= Gm::INVS, "the output stage fits the digit planes");
  {
    const double bz = p.bias ? (double)p.bias[grp * p.F + f0 + 16 * ft + r16] : 0.0;
#pragma unroll
    for (int i = 0; i < NTW; i++)
#pragma unroll
      for (int v = 0; v < 4; v++) ostage[(16 * ft + r16) * OS + 16 * (pg + PG * i) + 4 * q + v] = (float)(acc[i][v] + bz);
    if (tid < TP) {
      const int pi = p0 + tid, img = pi / OHW, rem = pi - img * OHW;
      pxoff[tid] = pi < p.P ? (img * G + grp) * p.F * OHW + rem : -1;
    }
  }
  __syncthreads();
  for (int idx = tid; idx < TF * TP; idx += SI8_THREADS) {
    const int fl = idx / TP, px = idx - fl * TP, po = pxoff[px];
    if (po >= 0) store_stream(p.O + (int64_t)po + (int64_t)(f0 + fl) * OHW, ostage[fl * OS + px]);
  }
}

}  // namespace tc355
