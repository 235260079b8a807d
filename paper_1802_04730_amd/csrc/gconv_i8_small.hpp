// Grouped convolution (Section 7, listing gconv) on the int8 matrix core for SMALL images: C = F = 16 channels per
// group, a 3 x 3 filter and a compile-time H x W (the paper's table shape (32,32,16,16,14,14)).  Arithmetic, digit
// layout and MFMA operand layout are those of gconv_i8.hpp (block scaling to 0x7F7F7F7E, four signed 8-bit digits, the
// 10 digit products with k + l >= 3 summed exactly in int32, one rounding to fp32); the blocks here are one filter
// row and one whole (image, group) block of 16 planes.
//
// Work split: a workgroup takes four images of one group at a time, one per wavefront, so that the four share one
// filter bank; everything else is private to the wavefront (its image's digit planes in LDS, its maximum, its
// outputs), and the wavefronts of a workgroup meet only where the filter bank changes.  The H x W image is small
// enough that a wavefront holds it whole: [4 digit planes][pixel][16 channels] bytes.  The OH x OW output pixels are
// numbered row-major and cut into tiles of 16 (144 = 9 tiles for 14 x 14: none is padded); a lane's B operand for
// (tile, kh) is the 16-byte record of pixel (h + kh, w + kw) of its own output pixel, so every (tile, kh) costs four
// LDS reads for 10 MFMAs.  The next image is fetched into registers while the current one is contracted.
// A launch at the paper's shape is one wave of workgroups, so the filter-bank setup is on its critical path and is kept
// short: 16 neighbouring lanes take one filter row, each one channel's 9 taps (loaded before the image is sliced),
// share the row's maximum through cross-lane moves and write their digit bytes straight into the records: no fp32
// copy in LDS, one barrier.
#pragma once
#include "gconv_i8.hpp"

namespace tc355 {

struct GconvI8SmallArgs {
  const float* I;
  const float* W1;
  const float* bias;  // or nullptr
  float* O;
  int G, N;           // N is a multiple of 4
};

template <int H, int W>
struct GconvI8SmallGeom {
  static constexpr int C = 16, F = 16, KH = 3, KW = 3;
  static constexpr int OH = H - KH + 1, OW = W - KW + 1;
  static constexpr int NPX = H * W, NOUT = OH * OW;
  static constexpr int TILES = (NOUT + 15) / 16;
  static constexpr int PLANE = NPX * 16;                     // bytes of one digit plane
  static constexpr int IMG = 4 * PLANE;                      // bytes of one wavefront's image
  static constexpr int NUNIT = NPX;                          // staging units of 4 channels x 4 pixels: (NPX / 4) * 4
  static constexpr int ROUNDS = (NUNIT + WAVE - 1) / WAVE;   // units per lane
  static constexpr int BANK = KH * 4 * WAVE * 16 + F * 4;    // the filter bank's digit records, then the filter rows' maxima
  static constexpr int LDS_BYTES = WAVES_PER_WG * IMG + BANK;
  static_assert(NPX % 4 == 0, "a channel plane is a whole number of 16-byte pieces");
  static_assert(3 * PLANE + ((H - 1) * W + W) * 16 < 65536, "LDS immediates out of range");
};

// MIND: the lowest digit diagonal k + l that is kept: 2 (13 products: what the library uses unless told that 10
// will do) or 3 (10 products).  The kernel's time is launch, cold start and set-up; the products hardly show.
template <int H, int W, int MIND = 2>
__global__ __launch_bounds__(WG_THREADS, 2) void gconv_i8_small_kernel(GconvI8SmallArgs p) {
  static_assert(MIND == 2 || MIND == 3, "13 or 10 digit products");
  using Gm = GconvI8SmallGeom<H, W>;
  constexpr int C = Gm::C, F = Gm::F, KH = Gm::KH, KW = Gm::KW, OW = Gm::OW, NPX = Gm::NPX, NOUT = Gm::NOUT,
                TILES = Gm::TILES, PLANE = Gm::PLANE, ROUNDS = Gm::ROUNDS;
  constexpr int WN = F * C * KH * KW, WPT = KH * KW;
  static_assert(F * C == WG_THREADS, "bank setup: one (filter row, channel) per thread");
  extern __shared__ __attribute__((aligned(16))) char gs_lds[];

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int kwq = q < KW ? q : KW - 1;  // slot group 3 is padding: it re-reads kw = 2 against zero weights
  char* img = gs_lds + wave * Gm::IMG;                       // this wavefront's digit planes
  char* arec = gs_lds + WAVES_PER_WG * Gm::IMG;
  unsigned* rowmax = reinterpret_cast<unsigned*>(arec + KH * 4 * WAVE * 16);  // largest magnitude of every filter row

  // this workgroup's run of iterations [u, u1); iteration = (group g, images 4j .. 4j+3), group-major
  const int per_group = p.N / WAVES_PER_WG;
  const unsigned iters = (unsigned)(p.G * per_group);
  unsigned u = iters * blockIdx.x / gridDim.x;
  const unsigned u1 = iters * (blockIdx.x + 1) / gridDim.x;
  if (u >= u1) return;

  // byte offset of this lane's B record for (tile t, kh = 0) inside a digit plane; pixels past the end repeat the last one
  int boff[TILES];
#pragma unroll
  for (int t = 0; t < TILES; t++) {
    const int px = min(16 * t + r16, NOUT - 1), h = px / OW, w = px - h * OW;
    boff[t] = (h * W + w + kwq) * 16;
  }

  // ---- staging units of this lane: unit = 4 channels (group cg) x 4 consecutive pixels (quad px4), unit = 4*px4 + cg
  f4 pre[ROUNDS][4];
  auto fetch = [&](int g, int n) {
    const float* src = p.I + ((int64_t)n * p.G + g) * (C * NPX);
#pragma unroll
    for (int r = 0; r < ROUNDS; r++) {
      const int unit = min(lane + r * WAVE, Gm::NUNIT - 1), cg = unit & 3, px4 = unit >> 2;
#pragma unroll
      for (int c = 0; c < 4; c++) pre[r][c] = *reinterpret_cast<const f4*>(src + (4 * cg + c) * NPX + 4 * px4);
    }
  };
  {
    const int g = (int)(u / per_group), n = (int)(u % per_group) * WAVES_PER_WG + wave;
    fetch(g, n);
  }

  i4 a[KH][4];     // a[kh][k]: digit k of W1[g][r16][c = byte][kh][kw = q], zeros for q = 3
  double fa[4];    // 2^24 / scale of filter row 4q + v (NaN if the row holds Inf/NaN)
  float bz[4];     // bias of filter row 4q + v
  int g_bank = -1;
  for (; u < u1; u++) {
    const int g = (int)(u / per_group), n = (int)(u % per_group) * WAVES_PER_WG + wave;
    // ---- a new group: this thread's share of the filter bank, the 9 taps of channel tid % 16 of filter row tid / 16
    const bool new_bank = g != g_bank;  // uniform over the workgroup
    float wv[WPT];
    if (new_bank) {
      const float* src = p.W1 + (int64_t)g * WN + tid * WPT;
#pragma unroll
      for (int j = 0; j < WPT; j++) wv[j] = src[j];
    }

    // ---- largest magnitude of the image block (this wavefront only)
    int mp = 0;
    unsigned mn = 0;
#pragma unroll
    for (int r = 0; r < ROUNDS; r++)
#pragma unroll
      for (int c = 0; c < 4; c++) {
        mp = i8_max3(mp, __float_as_int(pre[r][c][0]), __float_as_int(pre[r][c][1]));
        mn = i8_max3(mn, __float_as_uint(pre[r][c][0]), __float_as_uint(pre[r][c][1]));
        mp = i8_max3(mp, __float_as_int(pre[r][c][2]), __float_as_int(pre[r][c][3]));
        mn = i8_max3(mn, __float_as_uint(pre[r][c][2]), __float_as_uint(pre[r][c][3]));
      }
    const unsigned m = (unsigned)__builtin_amdgcn_readfirstlane((int)i8_wave_max(max((unsigned)mp, mn & 0x7fffffffu)));

    // ---- slice and stage: digit plane k, record of pixel pi at byte k*PLANE + 16*pi, channels 4cg.. at +4cg
    {
      const double sv = i8_scale(m);
      const double scale = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(sv)),
                                            __builtin_amdgcn_readfirstlane(__double2loint(sv)));
#pragma unroll
      for (int r = 0; r < ROUNDS; r++) {
        const int unit = lane + r * WAVE, cg = unit & 3, px4 = unit >> 2;
        if (unit < Gm::NUNIT) {
#pragma unroll
          for (int e = 0; e < 4; e++) {
            int d[4] = {i8_fixed<0x00808080>(pre[r][0][e], scale), i8_fixed<0x00808080>(pre[r][1][e], scale),
                        i8_fixed<0x00808080>(pre[r][2][e], scale), i8_fixed<0x00808080>(pre[r][3][e], scale)}, y[4];
            i8_transpose4(d, y);
#pragma unroll
            for (int k = 0; k < 4; k++)
              *reinterpret_cast<int*>(img + k * PLANE + 16 * (4 * px4 + e) + 4 * cg) = k < 3 ? y[k] ^ (int)0x80808080 : y[k];
          }
        }
      }
    }
    // ---- filter bank -> A operands: record (kh, k) of lane (r16, q) at arec + ((kh*4 + k)*64 + lane)*16 holds digit k
    // of W1[g][r16][channel = byte][kh][kw = q]; q = 3 is padding and holds zeros
    if (new_bank) {
      g_bank = g;
      __syncthreads();  // a slower wavefront may still be reading the records of the last bank
      const int row = tid >> 4, ch = tid & 15;
      unsigned mw = 0;
#pragma unroll
      for (int j = 0; j < WPT; j++) mw = max(mw, __float_as_uint(wv[j]) & 0x7fffffffu);
      int mv = (int)mw;  // sign cleared: signed and unsigned order agree
      mv = max(mv, __builtin_amdgcn_update_dpp(mv, mv, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
      mv = max(mv, __builtin_amdgcn_update_dpp(mv, mv, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
      mv = max(mv, __builtin_amdgcn_update_dpp(mv, mv, 0x141, 0xF, 0xF, false));  // row_half_mirror
      mv = max(mv, __builtin_amdgcn_update_dpp(mv, mv, 0x140, 0xF, 0xF, false));  // row_mirror: the row's 16 lanes
      if (ch == 0) rowmax[row] = (unsigned)mv;
      const double sa = i8_scale((unsigned)mv);  // mv = max|w| over the filter row
#pragma unroll
      for (int t = 0; t < WPT; t++) {
        const int d = i8_fixed<0x00808080>(wv[t], sa) ^ 0x00808080;  // byte k = digit k
#pragma unroll
        for (int k = 0; k < 4; k++)
          arec[(((t / KW) * 4 + k) * WAVE + 16 * (t % KW) + row) * 16 + ch] = (char)(d >> (8 * k));
      }
      if (tid < KH * 4 * 16)  // the padding records
        *reinterpret_cast<i4*>(arec + ((tid >> 4) * WAVE + 16 * KW + (tid & 15)) * 16) = i4{0, 0, 0, 0};
      __syncthreads();
#pragma unroll
      for (int kh = 0; kh < KH; kh++)
#pragma unroll
        for (int k = 0; k < 4; k++) a[kh][k] = *reinterpret_cast<const i4*>(arec + ((kh * 4 + k) * WAVE + lane) * 16);
#pragma unroll
      for (int v = 0; v < 4; v++) {
        fa[v] = 16777216.0 * i8_inverse_scale(rowmax[4 * q + v]);
        bz[v] = p.bias ? p.bias[g * F + 4 * q + v] : 0.f;
      }
    }
    // the next image of this wavefront, fetched while this one is contracted
    if (u + 1 < u1) {
      const unsigned un = u + 1;
      fetch((int)(un / per_group), (int)(un % per_group) * WAVES_PER_WG + wave);
    }
    const double invb = i8_inverse_scale(m);
    double fo[4];
#pragma unroll
    for (int v = 0; v < 4; v++) fo[v] = fa[v] * invb;

    // ---- contract: LDS operations of one wavefront execute in order, so its reads see the records staged above
    float* dst = p.O + ((int64_t)n * p.G + g) * (F * NOUT);
    const char* lbase = img;
#pragma unroll
    for (int t = 0; t < TILES; t++) {
      constexpr int ND = 7 - MIND, NP = MIND == 3 ? 10 : 13;
      i4 acc[ND];  // diagonals k + l = MIND .. 6
#pragma unroll
      for (int d = 0; d < ND; d++) acc[d] = i4{0, 0, 0, 0};
#pragma unroll
      for (int kh = 0; kh < KH; kh++) {
        i4 b[4];
#pragma unroll
        for (int l = 0; l < 4; l++) b[l] = *reinterpret_cast<const i4*>(lbase + boff[t] + l * PLANE + kh * W * 16);
        constexpr int PK[13] = {3, 3, 3, 3, 2, 2, 2, 1, 1, 0, 2, 1, 0};  // the last three: the diagonal k + l = 2
        constexpr int PL[13] = {3, 2, 1, 0, 3, 2, 1, 3, 2, 3, 0, 1, 2};
#pragma unroll
        for (int i = 0; i < NP; i++) acc[PK[i] + PL[i] - MIND] = mfma_i8(a[kh][PK[i]], b[PL[i]], acc[PK[i] + PL[i] - MIND]);
      }
      const int px = 16 * t + r16;
#pragma unroll
      for (int v = 0; v < 4; v++) {
        const int hi = acc[ND - 1][v] * 256 + acc[ND - 2][v];  // |.| < 2^30
        const int lo = acc[ND - 3][v] * 256 + acc[ND - 4][v];  // |.| < 2^31
        double rr = __builtin_fma((double)hi, 65536.0, (double)lo);  // sum_d P_d 256^(d-3), exact
        if constexpr (MIND == 2) rr = __builtin_fma((double)acc[0][v], 0.00390625, rr);
        const float o = (float)__builtin_fma(rr, fo[v], (double)bz[v]);
        if (px < NOUT) store_stream(dst + (4 * q + v) * NOUT + px, o);
      }
    }
  }
}

}  // namespace tc355
