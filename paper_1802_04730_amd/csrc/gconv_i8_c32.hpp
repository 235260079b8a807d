// Grouped convolution (Section 7, listing gconv) on the int8 matrix core for C = F = 32 channels per group, a 3 x 3
// filter and small compile-time H x W images (the paper's table shape (32,32,32,32,7,7)).  Arithmetic and digit
// layout are those of gconv_i8.hpp (block scaling to 0x7F7F7F7E, four signed 8-bit digits, the 10 digit products
// with k + l >= 3 summed exactly in int32, one rounding to fp32); the blocks are one filter row (288 weights) and
// one whole (image, group) block of 32 planes.
//
// v_mfma_i32_16x16x64_i8: rows = 16 filters (two filter tiles), columns = 16 output pixels (the OH x OW pixels
// numbered row-major and cut into tiles of 16), and the 64 reduction slots of one instruction are four slot groups
// of 16 channels: slot group sg = 4j + q of instruction j (q = lane / 16) carries tap sg / 2 = 3 kh + kw and channel
// half sg % 2.  The 9 taps x 2 halves fill 18 of the 20 slot groups of five instructions; the last two hold zero
// weights.  A lane's B operand for (pixel tile, j) is the 16-byte half record of its own output pixel shifted by the
// tap, so the image needs no im2col: it sits in LDS as [4 digit planes][pixel][32 channels] bytes.
//
// Work split: a workgroup of four wavefronts takes four images of one group at a time, one per wavefront; the filter
// bank (2 filter tiles x 5 instructions x 4 digits of A operands: too many for the register file) is sliced once per
// group into LDS records that all wavefronts read; everything else is private to a wavefront.  A launch at the
// paper's shape is one wave of workgroups, so the bank setup is on its critical path and is kept short: eight
// neighbouring lanes take one filter row, each 4 channels x 9 taps of it (36 consecutive floats: nine 16-byte loads,
// issued before the image is sliced), share the row's maximum through cross-lane moves, and write their digits
// straight into the records: no fp32 copy in LDS, no LDS reads, one barrier.
#pragma once
#include "gconv_i8.hpp"

namespace tc355 {

struct GconvI8C32Args {
  const float* I;
  const float* W1;
  const float* bias;  // or nullptr
  float* O;
  int G, N;           // N is a multiple of 4
};

template <int H, int W>
struct GconvI8C32Geom {
  static constexpr int NW = WAVES_PER_WG, NT = WG_THREADS;
  static constexpr int C = 32, F = 32, KH = 3, KW = 3, TAPS = KH * KW;
  static constexpr int OH = H - KH + 1, OW = W - KW + 1;
  static constexpr int NPX = H * W, NOUT = OH * OW;
  static constexpr int PT = (NOUT + 15) / 16;               // pixel tiles
  static constexpr int FT = F / 16;                         // filter tiles
  static constexpr int NJ = (2 * TAPS + 3) / 4;             // instructions per (filter tile, pixel tile, digit pair): 5
  static constexpr int PLANE = NPX * C;                     // bytes of one digit plane
  static constexpr int IMG = 4 * PLANE;                     // bytes of one wavefront's image
  static constexpr int NUNIT = NPX * (C / 4);               // staging units: one pixel x 4 channels
  static constexpr int ROUNDS = (NUNIT + WAVE - 1) / WAVE;
  static constexpr int AREC = FT * NJ * 4 * WAVE * 16;      // A operand records: [ft][j][digit][lane] x 16 bytes
  static constexpr int LDS_BYTES = NW * IMG + AREC + F * 4;  // + the filter rows' maxima
  static constexpr int TPR = NT / F;                        // threads that share a filter row: 8
  static constexpr int EPT = C * TAPS / TPR;                // elements of the row per such thread: 4 channels x 9 taps
  static_assert(TPR == 8 && EPT == 4 * TAPS && EPT % 4 == 0, "bank setup: a thread takes 4 channels of one filter row");
  static_assert(FT * 4 * 16 * 2 == NT && 2 * TAPS + 2 == 4 * NJ, "one padding record per thread");
  static_assert(3 * PLANE + NPX * C < 65536, "LDS immediates out of range");
};

// MIND: the lowest digit diagonal k + l that is kept: 2 (13 products: what the library uses unless told that 10
// will do) or 3 (10 products).
template <int H, int W, int MIND = 2>
__global__ __launch_bounds__(WG_THREADS, 2) void gconv_i8_c32_kernel(GconvI8C32Args p) {
  static_assert(MIND == 2 || MIND == 3, "13 or 10 digit products");
  using Gm = GconvI8C32Geom<H, W>;
  constexpr int NW = Gm::NW;
  constexpr int C = Gm::C, F = Gm::F, KW = Gm::KW, TAPS = Gm::TAPS, OW = Gm::OW, NPX = Gm::NPX, NOUT = Gm::NOUT,
                PT = Gm::PT, FT = Gm::FT, NJ = Gm::NJ, PLANE = Gm::PLANE, ROUNDS = Gm::ROUNDS;
  extern __shared__ __attribute__((aligned(16))) char gc_lds[];

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  char* img = gc_lds + wave * Gm::IMG;                       // this wavefront's digit planes
  char* arec = gc_lds + NW * Gm::IMG;
  unsigned* rowmax = reinterpret_cast<unsigned*>(arec + Gm::AREC);  // largest magnitude of every filter row

  // this workgroup's run of iterations [u, u1); iteration = (group g, images NW i .. NW i + NW - 1), group-major
  const int per_group = p.N / NW;
  const unsigned iters = (unsigned)(p.G * per_group);
  unsigned u = iters * blockIdx.x / gridDim.x;
  const unsigned u1 = iters * (blockIdx.x + 1) / gridDim.x;
  if (u >= u1) return;

  // tap and channel half of this lane's slot group in instruction j; slot groups past the 18 real ones are padding
  int tapj[NJ], halfj[NJ];
  bool realj[NJ];
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const int sg = 4 * j + q;
    realj[j] = sg < 2 * TAPS;
    tapj[j] = min(sg >> 1, TAPS - 1);
    halfj[j] = sg & 1;
  }
  // byte offset of this lane's B half record for (pixel tile t, instruction j) inside a digit plane
  int boff[PT][NJ];
#pragma unroll
  for (int t = 0; t < PT; t++) {
    const int px = min(16 * t + r16, NOUT - 1), h = px / OW, w = px - h * OW;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
      const int kh = tapj[j] / KW, kw = tapj[j] - kh * KW;
      boff[t][j] = ((h + kh) * W + w + kw) * C + 16 * halfj[j];
    }
  }

  // ---- staging units of this lane: unit = (channel group cg of 4, pixel px), pixels fastest (coalesced 4-byte loads)
  float pre[ROUNDS][4];
  auto fetch = [&](int g, int n) {
    const float* src = p.I + ((int64_t)n * p.G + g) * (C * NPX);
#pragma unroll
    for (int r = 0; r < ROUNDS; r++) {
      const int unit = min(lane + r * WAVE, Gm::NUNIT - 1), cg = unit / NPX, px = unit - cg * NPX;
#pragma unroll
      for (int c = 0; c < 4; c++) pre[r][c] = src[(4 * cg + c) * NPX + px];
    }
  };
  fetch((int)(u / per_group), (int)(u % per_group) * NW + wave);

  double fa[FT][4];  // 2^24 / scale of filter row 16 ft + 4q + v (NaN if the row holds Inf/NaN)
  float bz[FT][4];   // bias of that row
  int g_bank = -1;
  for (; u < u1; u++) {
    const int g = (int)(u / per_group), n = (int)(u % per_group) * NW + wave;
    // ---- a new group: this thread's share of the filter bank, 4 channels x 9 taps of filter row tid / 8
    const bool new_bank = g != g_bank;  // uniform over the workgroup
    f4 wv[Gm::EPT / 4];
    if (new_bank) {
      const f4* src = reinterpret_cast<const f4*>(p.W1 + ((int64_t)g * F + tid / Gm::TPR) * (C * TAPS) + (tid % Gm::TPR) * Gm::EPT);
#pragma unroll
      for (int r = 0; r < Gm::EPT / 4; r++) wv[r] = src[r];
    }

    // ---- largest magnitude of the image block (this wavefront only)
    int mp = 0;
    unsigned mn = 0;
#pragma unroll
    for (int r = 0; r < ROUNDS; r++) {
      mp = i8_max3(mp, __float_as_int(pre[r][0]), __float_as_int(pre[r][1]));
      mn = i8_max3(mn, __float_as_uint(pre[r][0]), __float_as_uint(pre[r][1]));
      mp = i8_max3(mp, __float_as_int(pre[r][2]), __float_as_int(pre[r][3]));
      mn = i8_max3(mn, __float_as_uint(pre[r][2]), __float_as_uint(pre[r][3]));
    }
    const unsigned m = (unsigned)__builtin_amdgcn_readfirstlane((int)i8_wave_max(max((unsigned)mp, mn & 0x7fffffffu)));

    // ---- slice and stage: digit plane k, record of pixel px at byte k*PLANE + 32*px, channels 4cg.. at +4cg
    {
      const double sv = i8_scale(m);
      const double scale = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(sv)),
                                            __builtin_amdgcn_readfirstlane(__double2loint(sv)));
#pragma unroll
      for (int r = 0; r < ROUNDS; r++) {
        const int unit = lane + r * WAVE, cg = unit / NPX, px = unit - cg * NPX;
        if (unit < Gm::NUNIT) {
          int d[4] = {i8_fixed<0x00808080>(pre[r][0], scale), i8_fixed<0x00808080>(pre[r][1], scale),
                      i8_fixed<0x00808080>(pre[r][2], scale), i8_fixed<0x00808080>(pre[r][3], scale)}, y[4];
          i8_transpose4(d, y);
#pragma unroll
          for (int k = 0; k < 4; k++)
            *reinterpret_cast<int*>(img + k * PLANE + C * px + 4 * cg) = k < 3 ? y[k] ^ (int)0x80808080 : y[k];
        }
      }
    }
    // ---- filter bank -> A operand records in LDS: record (ft, j, k) of lane (r16, q) at
    // arec + (((ft*NJ + j)*4 + k)*64 + lane)*16 holds digit k of filter 16 ft + r16, tap and channel half of slot
    // group 4 j + q, 16 channels.  This thread has filter row 16 ft + r16' = tid / 8 and channels 4 part ..
    if (new_bank) {
      g_bank = g;
      __syncthreads();  // every wavefront is done with the records of the last group
      const int row = tid / Gm::TPR, part = tid % Gm::TPR;
      const float* w = reinterpret_cast<const float*>(wv);  // [channel c of 4][tap]
      unsigned m = 0;
#pragma unroll
      for (int i = 0; i < Gm::EPT; i++) m = max(m, __float_as_uint(w[i]) & 0x7fffffffu);
      int mv = (int)m;  // sign cleared: signed and unsigned order agree
      mv = max(mv, __builtin_amdgcn_update_dpp(mv, mv, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
      mv = max(mv, __builtin_amdgcn_update_dpp(mv, mv, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
      mv = max(mv, __builtin_amdgcn_update_dpp(mv, mv, 0x141, 0xF, 0xF, false));  // row_half_mirror: the row's 8 lanes
      if (part == 0) rowmax[row] = (unsigned)mv;
      const double sa = i8_scale((unsigned)mv);
      char* rec = arec + ((row >> 4) * NJ * 4 * WAVE + (row & 15)) * 16 + 4 * (part & 3);
      const int half = part >> 2;
#pragma unroll
      for (int t = 0; t < TAPS; t++) {
        int d[4], y[4];
#pragma unroll
        for (int c = 0; c < 4; c++) d[c] = i8_fixed<0x00808080>(w[c * TAPS + t], sa) ^ 0x00808080;
        i8_transpose4(d, y);
        // slot group 2 t + half = 4 j + q: only q depends on the thread
        const int j = (2 * t) / 4, q0 = (2 * t) % 4;
#pragma unroll
        for (int k = 0; k < 4; k++)
          *reinterpret_cast<int*>(rec + ((j * 4 + k) * WAVE + 16 * (q0 + half)) * 16) = y[k];
      }
      {  // the two slot groups past the 18 real ones (instruction NJ - 1, q = 2 and 3) hold zero weights
        const int ft = tid >> 7, k = (tid >> 5) & 3, qq = 2 + ((tid >> 4) & 1);
        *reinterpret_cast<i4*>(arec + (((ft * NJ + NJ - 1) * 4 + k) * WAVE + 16 * qq + (tid & 15)) * 16) = i4{0, 0, 0, 0};
      }
      __syncthreads();  // records and row maxima complete
#pragma unroll
      for (int ft = 0; ft < FT; ft++)
#pragma unroll
        for (int v = 0; v < 4; v++) {
          fa[ft][v] = 16777216.0 * i8_inverse_scale(rowmax[16 * ft + 4 * q + v]);
          bz[ft][v] = p.bias ? p.bias[g * F + 16 * ft + 4 * q + v] : 0.f;
        }
    }
    // the next image of this wavefront, fetched while this one is contracted
    if (u + 1 < u1) {
      const unsigned un = u + 1;
      fetch((int)(un / per_group), (int)(un % per_group) * NW + wave);
    }
    const double invb = i8_inverse_scale(m);

    // ---- contract: LDS operations of one wavefront execute in order, so its reads see the records staged above
    float* dst = p.O + ((int64_t)n * p.G + g) * (F * NOUT);
#pragma unroll
    for (int ft = 0; ft < FT; ft++) {
      i4 a[NJ][4];
#pragma unroll
      for (int j = 0; j < NJ; j++)
#pragma unroll
        for (int k = 0; k < 4; k++)
          a[j][k] = *reinterpret_cast<const i4*>(arec + (((ft * NJ + j) * 4 + k) * WAVE + lane) * 16);
#pragma unroll
      for (int t = 0; t < PT; t++) {
        constexpr int ND = 7 - MIND, NP = MIND == 3 ? 10 : 13;
        i4 acc[ND];  // diagonals k + l = MIND .. 6
#pragma unroll
        for (int d = 0; d < ND; d++) acc[d] = i4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NJ; j++) {
          i4 b[4];
#pragma unroll
          for (int l = 0; l < 4; l++) b[l] = *reinterpret_cast<const i4*>(img + boff[t][j] + l * PLANE);
          constexpr int PK[13] = {3, 3, 3, 3, 2, 2, 2, 1, 1, 0, 2, 1, 0};  // the last three: the diagonal k + l = 2
          constexpr int PL[13] = {3, 2, 1, 0, 3, 2, 1, 3, 2, 3, 0, 1, 2};
#pragma unroll
          for (int i = 0; i < NP; i++) acc[PK[i] + PL[i] - MIND] = mfma_i8(a[j][PK[i]], b[PL[i]], acc[PK[i] + PL[i] - MIND]);
        }
        const int px = 16 * t + r16;
#pragma unroll
        for (int v = 0; v < 4; v++) {
          // sum_d P_d 256^(d-3), exact.  (With 288 terms per output 256 * P_4 + P_3 can pass 2^31, so the diagonals
          // are combined in fp64 rather than pairwise in int32 as in the 16-channel kernels.)
          double rr = __builtin_fma((double)acc[ND - 1][v], 16777216.0,
                                    __builtin_fma((double)acc[ND - 2][v], 65536.0,
                                                  __builtin_fma((double)acc[ND - 3][v], 256.0, (double)acc[ND - 4][v])));
          if constexpr (MIND == 2) rr = __builtin_fma((double)acc[0][v], 0.00390625, rr);
          const float o = (float)__builtin_fma(rr, fa[ft][v] * invb, (double)bz[ft][v]);
          if (px < NOUT) store_stream(dst + (16 * ft + 4 * q + v) * NOUT + px, o);
        }
      }
    }
  }
}

}  // namespace tc355
