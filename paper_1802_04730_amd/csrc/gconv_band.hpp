// Grouped convolution (Section 7, listing gconv), fastest path: channel counts
// that fit the matrix core (C % 4 == 0, F == 16), small filter, image width known
// at compile time.
//
//   O(n,g,o,h,w) = sum_{i,kh,kw} I(n,g,i,h+kh,w+kw) * W1(g,o,i,kh,kw) + bias(g*F+o)
//
// On this chip a vector-ALU instruction and an fp64 MFMA of the same wavefront
// slot do not overlap, so every widening or address add inside the contraction
// loop is paid in matrix-pipe time.  This kernel therefore moves all of that
// out of the loop:
//   * one workgroup (4 wavefronts) walks one (image, group) pair band by band;
//     a band is ROWS output rows = ROWS*OW pixels = 16-pixel tiles dealt evenly
//     to the wavefronts;
//   * the band's input rows (ROWS+KH-1 rows, all C channels) sit in LDS already
//     WIDENED to fp64 (each element is widened once when staged and then read
//     KH*KW times), plane stride = 16 (mod 32) doubles so the four k slots of a
//     wavefront hit disjoint banks;
//   * the group's filter bank sits in registers as fp64 MFMA A operands for the
//     lifetime of the workgroup;
//   * the reduction is consumed in the order (kh, kw, c/4) with k slot q carrying
//     channel 4*(c/4)+q, so every B operand is one 8-byte LDS read at
//     "lane base + compile-time immediate" that feeds the MFMA directly;
//   * the tiles of a wavefront advance together step by step, and the LDS reads
//     of the next step are issued before the MFMAs of the current one;
//   * the next band is fetched from global memory into registers while the
//     current one is contracted, one 16-byte load every few MFMA steps: issued
//     as one burst, the loads of all workgroups pile up in the memory pipeline
//     and block the issuing wavefronts for ~10 us per band (measured).
// Two workgroups fit per compute unit (2 x 74 KiB of LDS).  The accumulators start from the bias (fp64), so the epilogue is the single rounding.
#pragma once
#include <type_traits>

#include "tc355_device.hpp"

namespace tc355 {

struct GconvBandArgs {
  const float* I;
  const float* W1;
  const float* bias;  // or nullptr
  float* O;
  int G, H;
};

template <int C, int KH, int KW, int W, int ROWS>
struct GconvBandGeom {
  static constexpr int F = 16;
  static constexpr int OW = W - KW + 1;
  static constexpr int IN_ROWS = ROWS + KH - 1;
  static constexpr int LEN = IN_ROWS * W;                  // floats per channel plane of a band
  static constexpr int PS = ((LEN + 31 - 16) / 32) * 32 + 16;  // plane stride in doubles, = 16 (mod 32), >= LEN
  static constexpr int LDS_BYTES = C * PS * 8;
  static constexpr int TILES = (ROWS * OW + 15) / 16;      // 16-pixel tiles per band
  static constexpr int TP = (TILES + WAVES_PER_WG - 1) / WAVES_PER_WG;
  static constexpr int NS = KH * KW * (C / 4);             // MFMA steps per tile
  static constexpr int LEN4 = (LEN + 3) / 4;
  static constexpr int NLD = (C * LEN4 + WG_THREADS - 1) / WG_THREADS;  // 16-byte loads per thread and band
  static_assert(PS >= LEN, "plane stride too small");
  static_assert((4 * (C / 4 - 1) * PS + (KH - 1) * W + KW - 1) * 8 < 65536, "LDS immediates out of range");
};

template <int C, int KH, int KW, int W, int ROWS, int MINW>
__global__ __launch_bounds__(WG_THREADS, MINW) void gconv_band_kernel(GconvBandArgs p) {
  using Gm = GconvBandGeom<C, KH, KW, W, ROWS>;
  constexpr int F = Gm::F, OW = Gm::OW, PS = Gm::PS, NS = Gm::NS, LEN = Gm::LEN, LEN4 = Gm::LEN4, NLD = Gm::NLD;
  extern __shared__ __attribute__((aligned(16))) double band[];  // [C][PS]

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int64_t ng = blockIdx.x;  // n*G + g
  const int g = (int)(ng % p.G);
  const int H = p.H, OH = H - KH + 1;
  const int npix = OH * OW;
  const int nbands = (OH + ROWS - 1) / ROWS;
  const int64_t plane = (int64_t)H * W;
  const float* src = p.I + ng * C * plane;
  float* dst = p.O + ng * (int64_t)F * npix;
  const bool vec_ok = (plane & 3) == 0 && ((ROWS * W) & 3) == 0;  // every band start is 16-byte aligned

  // ---- band fetch (global -> registers) and staging (registers -> fp64 LDS)
  f4 pre[NLD];
  // one 16-byte unit (index j of this thread) of band b: global -> register
  auto fetch_one = [&](int b, int j) {
    const int h0 = b * ROWS;
    const int avail = (H - h0) * W;  // floats of each plane from row h0 to the end of the image
    const int idx = tid + j * WG_THREADS;
    const int c = idx / LEN4, i = (idx - c * LEN4) * 4;
    f4 v = {0.f, 0.f, 0.f, 0.f};
    if (idx < C * LEN4) {
      const float* s = src + c * plane + (int64_t)h0 * W + i;
      if (vec_ok) {
        if (i + 3 < avail) v = *reinterpret_cast<const f4*>(s);
      } else {
#pragma unroll
        for (int e = 0; e < 4; e++)
          if (i + e < avail && i + e < LEN) v[e] = s[e];
      }
    }
    pre[j] = v;
  };
#pragma unroll
  for (int j = 0; j < NLD; j++) fetch_one(0, j);  // first band: in flight while the filter bank is set up

  // ---- filter bank -> registers: a[s] = W1[g][r16][4*c4+q][kh][kw], s = (kh*KW+kw)*(C/4)+c4.
  // The bank of a group is one contiguous block of F*C*KH*KW floats: fetch it with coalesced
  // loads, park it in the (still unused) band area of LDS, and let every lane pick its values.
  double a[NS];
  {
    constexpr int WN = F * C * KH * KW;
    float* wl = reinterpret_cast<float*>(band);
    const float* wg = p.W1 + (int64_t)g * WN;
    for (int i = tid; i < WN; i += WG_THREADS) wl[i] = wg[i];
    __syncthreads();
    const float* wp = wl + (r16 * C + q) * (KH * KW);
#pragma unroll
    for (int kk = 0; kk < KH * KW; kk++)
#pragma unroll
      for (int c4 = 0; c4 < C / 4; c4++) a[kk * (C / 4) + c4] = (double)wp[4 * c4 * (KH * KW) + kk];
    // the first band is staged only after the __syncthreads() at the top of the band loop
  }
  double bz[4];
#pragma unroll
  for (int v = 0; v < 4; v++) bz[v] = p.bias ? (double)p.bias[g * F + d_row(q, v)] : 0.0;

  auto stage = [&]() {
#pragma unroll
    for (int j = 0; j < NLD; j++) {
      const int idx = tid + j * WG_THREADS;
      const int c = idx / LEN4, i = (idx - c * LEN4) * 4;
      if (idx < C * LEN4) {
        double* d = band + c * PS + i;  // PS and i are even: 16-byte aligned pairs
        dbl2 lo = {(double)pre[j][0], (double)pre[j][1]}, hi = {(double)pre[j][2], (double)pre[j][3]};
        *reinterpret_cast<dbl2*>(d) = lo;
        *reinterpret_cast<dbl2*>(d + 2) = hi;  // PS is a multiple of 16 >= LEN, so i + 3 < PS
      }
    }
  };

  for (int b = 0; b < nbands; b++) {
    __syncthreads();  // everyone has finished reading the previous band
    stage();
    __syncthreads();
    const bool more = b + 1 < nbands;  // the next band is fetched piecemeal between the MFMA steps below:
    // issued in one burst, the loads of all workgroups pile up in the memory pipeline and the
    // issuing wavefronts sit blocked for ~10 us; spread out, they vanish behind the MFMAs

    const int P0 = b * ROWS * OW;
    // Tiles of the band are dealt to the wavefronts round-robin: tile id = 4*t + wr.  Every wavefront
    // gets FULL = TILES/4 of them; the first TILES%4 ranks get one more.  The rank wr of a wavefront
    // rotates with the band number, so over four bands every SIMD does the same amount of work.
    constexpr int TILES = Gm::TILES, FULL = TILES / WAVES_PER_WG, REM = TILES % WAVES_PER_WG;
    const int wr = (wave + b) & (WAVES_PER_WG - 1);
    auto tile_ptr = [&](int tile) {
      const int px = min(min(P0 + tile * 16 + r16, npix - 1) - P0, ROWS * OW - 1);  // clamp a ragged last band
      return band + q * PS + (px / OW) * W + (px % OW);
    };
    // TN tiles advance together, one reduction step at a time; the LDS reads of step s+1 are issued
    // before the MFMAs of step s.  FETCH: units [j0, j0+NJ) of the next band are fetched between steps.
    auto group = [&](auto tn_c, int t_first, auto j0_c, auto nj_c) {
      constexpr int TN = decltype(tn_c)::value, J0 = decltype(j0_c)::value, NJ = decltype(nj_c)::value;
      constexpr int NJD = NJ > 0 ? NJ : 1;  // (keeps the unused branch free of a division by zero)
      constexpr int EVERY = NJ > 0 ? (NS / NJD > 0 ? NS / NJD : 1) : NS + 1;
      const double* bp[TN];
      d4 acc[TN];
      double bcur[TN], bnxt[TN];
#pragma unroll
      for (int t = 0; t < TN; t++) {
        bp[t] = tile_ptr(4 * (t_first + t) + wr);
        acc[t] = d4{bz[0], bz[1], bz[2], bz[3]};  // start from the bias: one add less per output
        bcur[t] = bp[t][0];
      }
#pragma unroll
      for (int s = 0; s < NS; s++) {
        if (NJ > 0 && s % EVERY == EVERY / 2 && s / EVERY < NJ && more) fetch_one(b + 1, J0 + s / EVERY);
        if (s + 1 < NS) {
          const int kk = (s + 1) / (C / 4), c4 = (s + 1) % (C / 4);
          const int off = 4 * c4 * PS + (kk / KW) * W + (kk % KW);
#pragma unroll
          for (int t = 0; t < TN; t++) bnxt[t] = bp[t][off];
        }
        // pin the order "reads of step s+1, then MFMAs of step s": left alone, the compiler sinks
        // the reads below the MFMAs to save registers and the LDS latency lands on the matrix pipe
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < TN; t++) acc[t] = mfma_f64(a[s], bcur[t], acc[t]);
#pragma unroll
        for (int t = 0; t < TN; t++) bcur[t] = bnxt[t];
        // keep the compiler from hoisting every LDS read of the group to the top (register spills)
        __builtin_amdgcn_sched_barrier(0);
      }
      if (NJ > 0 && more) {  // units the loop had no step for
#pragma unroll
        for (int j = (NS - 1 - EVERY / 2) / EVERY + 1; j < NJ; j++) fetch_one(b + 1, J0 + j);
      }
#pragma unroll
      for (int t = 0; t < TN; t++) {
        const int pl = (4 * (t_first + t) + wr) * 16 + r16;  // pixel within the band
        if (pl < ROWS * OW && P0 + pl < npix) {
#pragma unroll
          for (int v = 0; v < 4; v++) store_stream(&dst[(int64_t)d_row(q, v) * npix + P0 + pl], (float)acc[t][v]);
        }
      }
    };
    using std::integral_constant;
    // FULL tiles in groups of at most 4 (bounds the live registers); the next band's NLD fetch units
    // are spread over the groups in proportion
    constexpr int G1 = FULL < 4 ? FULL : 4, G2 = FULL - G1 < 4 ? FULL - G1 : 4;
    static_assert(FULL >= 1 && FULL <= 8, "1..8 whole tiles per wavefront and band");
    constexpr int NJ1 = G2 > 0 ? (NLD * G1 + FULL - 1) / FULL : NLD;
    group(integral_constant<int, G1>{}, 0, integral_constant<int, 0>{}, integral_constant<int, NJ1>{});
    if constexpr (G2 > 0)
      group(integral_constant<int, G2>{}, G1, integral_constant<int, NJ1>{}, integral_constant<int, NLD - NJ1>{});
    if constexpr (REM > 0) {
      if (wr < REM) group(integral_constant<int, 1>{}, FULL, integral_constant<int, 0>{}, integral_constant<int, 0>{});
    }
  }
}

}  // namespace tc355
