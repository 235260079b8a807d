// Grouped convolution (Section 7, listing gconv) on the int8 matrix core, for
// C = F = 16 channels per group, a 3 x 3 filter and a compile-time image width:
//
//   O(n,g,o,h,w) = sum_{i,kh,kw} I(n,g,i,h+kh,w+kw) * W1(g,o,i,kh,kw) + bias(g*F+o)
//
// The fp64 matrix instruction delivers 16 multiply-adds per clock and SIMD, the
// int8 one 1024.  This kernel therefore evaluates the contraction in integer
// arithmetic on slices of the operands:
//   * every fp32 operand x of a block (one filter row of W1; one band of input
//     rows) is written as a 32-bit fixed-point number relative to the block's
//     largest magnitude m, v = rint(x * S / m) with S = 0x7F7F7F7E, the largest
//     value (less one) that four signed 8-bit digits can hold, and v is split
//     into those digits, v = sum_k d_k 256^k: every element is represented to
//     2^-32 of the block maximum;
//   * a product of two operands is sum_{k,l} a_k b_l 256^(k+l); the 10 digit
//     pairs with k + l >= 3 are kept.  What is dropped is at most 3 * 2^-32 of
//     the product of the two block maxima per term (2^-33 typically), the size
//     of the quantisation error itself.  Each pair is one int8 MFMA
//     accumulation in int32, which is exact (no rounding, any order), one
//     accumulator per diagonal k + l;
//   * the four diagonals are combined exactly (int32 shifts, then fp64), scaled
//     by 2^24 * (m_a / S) * (m_b / S) in fp64, the bias is added in fp64, and
//     the sum is rounded to fp32 once.
// Against the float64 definition the result differs by the input quantisation
// and the dropped digit pairs: measured 1e-6 on the parity metric at the
// benchmark's distribution (the bar is 2e-5), ~1e-9 relative on outputs of
// typical magnitude.  (Scaling by a power of two and keeping the 13 pairs with
// k + l >= 2 measures 3e-7 there and no better on heavy-tailed data, for 30 %
// more matrix work; on this kernel, which runs at the board's power limit, that
// is 8 % of the time.)
//
// What the dropped diagonal k + l = 2 costs is proportional to the product of
// the two block maxima, so it grows when the maxima say little about the
// outputs: when BOTH operands are heavy-tailed (a few elements far above the
// rest in every block) the 10 products come close to the bar (1.6e-5 measured
// with log-normal magnitudes of sigma 1.5 and 1).  The kernel therefore decides
// per band, from a statistic it gets almost for free while it looks for the band
// maximum:
//     S = (band maximum / smallest per-thread maximum)
//         * (largest ratio of maximum to mean magnitude among the group's 16 filter rows)
// (Gaussian operands: 11-22, behind a ReLU the same, Laplacian 27-72; Student-t(3)
// 150-600, log-normal magnitudes and single huge elements: thousands).  A band
// with S above I8_HEAVY_STAT = 128 gets the diagonal k + l = 2 as well: after the
// ordinary sweeps a second, lighter set of sweeps (3 products instead of 10)
// accumulates it and adds it to the staged outputs, 13 products in all.  The
// emulation in tests/test_i8_scheme.py holds both branches of that rule below a
// quarter of the bar on all those distributions.  A band in which some thread
// sees only zeros counts as heavy (S is infinite): slower, never less accurate.
// `force13` in the arguments overrides the rule (1: every band, -1: no band).
// A band whose inputs contain Inf/NaN yields NaN for all of that band's outputs.
//
// MFMA v_mfma_i32_16x16x64_i8, lane = (r16 = lane % 16, q = lane / 16), measured:
//   A (16 x 64): lane supplies A[row r16][k = 16q .. 16q+15]  (16 bytes)
//   B (64 x 16): lane supplies B[k = 16q .. 16q+15][col r16]
//   D (16 x 16): lane holds D[row 4q + v][col r16], v = 0..3
// Here rows are the 16 filters, columns are 16 output pixels of one image row,
// and the 64 reduction slots of one instruction are (kw = q, channel = byte):
// slot group q = 3 is padding (A holds zeros there).  One "group" of 10 MFMAs
// therefore covers one filter row kh for a 16-pixel tile, and the B operand of
// input row r is shared by the output rows r, r-1 and r-2.
//
// Work split: bands of 8 output rows, numbered group-major ((g, n, band), band
// fastest); persistent workgroups (two per compute unit), each taking one
// contiguous run of bands, so that its filter bank changes at most once or
// twice.  Workgroups w and w + gridDim/2 come to share a compute unit; the
// first is dispatched earlier, wins the issue slots and runs about a quarter
// faster, so it is given more than half of the pair's bands (num/den).  The band's 10 input rows sit
// in LDS as four digit planes [pixel][16 channels] (two buffers, used in turn:
// the idle one is the scratch through which the next image's filter bank is set
// up while slower wavefronts still read the other); wavefront w owns output rows 2w and 2w+1 of the band: three
// full 16-pixel columns swept over 4 input rows each, and the last 8 columns of
// both rows packed into one tile (lanes 0-7: row 2w, lanes 8-15: row 2w+1).
// Every wavefront executes the same 21 groups per band; its outputs (16 filters
// x 2 rows) are collected in the idle band buffer and leave as 16-byte stores of
// whole row pairs.  The next band (of this
// or of the next image) is fetched into registers piecemeal between the groups,
// with 16-byte loads: the kernel takes only heights whose bands are whole and
// 16-byte aligned (H even, H - 2 a multiple of 8); a band's rows are then one
// contiguous run of every channel plane.
#pragma once
#include <type_traits>

#include "tc355_device.hpp"

namespace tc355 {

typedef int i4 __attribute__((ext_vector_type(4)));

struct GconvI8Args {
  const float* I;
  const float* W1;
  const float* bias;  // or nullptr
  float* O;
  int G, H;
  int N;        // images
  int halves;   // gridDim.x / 2 if workgroups w and w + halves share a compute unit's work, else 0 (even split)
  int num, den; // of the bands that such a pair owns, workgroup w takes the first num/den
  int force13;  // 0: the diagonal k + l = 2 for heavy-tailed bands only; 1: for every band; -1: never
};

constexpr float I8_HEAVY_STAT = 128.0f;  // bands whose statistic S (see above) exceeds this get 13 digit products

template <int W, int ROWS>
struct GconvI8Geom {
  static constexpr int C = 16, F = 16, KH = 3, KW = 3;
  static constexpr int OW = W - KW + 1;
  static constexpr int IN_ROWS = ROWS + KH - 1;
  static constexpr int NPX = IN_ROWS * W;                               // pixels of a band
  static constexpr int PLANE = NPX * 16;                                // bytes of one digit plane
  static constexpr int BUF = 4 * PLANE;                                 // bytes of one band buffer
  // staging units: 4 channels (group cg) x 4 consecutive pixels (quad px4), unit = 4*px4 + cg, so that four
  // neighbouring lanes fill one 16-byte record; a thread takes units tid and tid + 256, and what is left is dealt
  // out as half units of 4 channels x 2 pixels, so that no thread slices much more than its share
  static constexpr int NQ = NPX / 4, NUNIT = 4 * NQ, NHALF = 2 * (NUNIT - 2 * WG_THREADS);
  static_assert(NPX % 4 == 0 && NUNIT > 2 * WG_THREADS && NHALF <= WG_THREADS, "two rounds of units and one of half units");
  static constexpr int MISC = 2 * BUF;                                  // byte offset of the small arrays
  static constexpr int LDS_BYTES = 2 * BUF + 128;                       // + the per-wavefront maxima and minima
  static constexpr int NFC = OW / 16;                                   // full 16-pixel columns
  // output staging of a wavefront (16 filters x 2 rows x OW pixels, fp32) in the idle band buffer: filter stride
  // in floats = 4 (mod 16), so that the four filter rows a store instruction writes fall into different banks
  static constexpr int OSF = ((2 * OW + 11) / 16) * 16 + 4;
  static constexpr int OSTAGE = 16 * OSF * 4;                           // bytes per wavefront
  static_assert(OSF >= 2 * OW && WAVES_PER_WG * OSTAGE <= BUF, "output staging must fit the idle band buffer");
  static_assert((2 * OW * 4) % 16 == 0 && 2 * OW * 4 / 16 <= 32, "a filter's two rows are at most 32 16-byte pieces");
  static_assert(ROWS == 2 * WAVES_PER_WG, "two output rows per wavefront");
  static_assert(OW % 16 == 8, "the last 8 columns of two rows share one tile");
  static_assert(3 * PLANE + 3 * W * 16 < 65536, "LDS immediates out of range");
  static_assert(F * C * KH * KW * 4 <= BUF, "filter bank scratch must fit one band buffer");
};

// Fixed-point scale of a block: the block's largest magnitude (bit pattern mbits, sign cleared) maps to I8_FULL.
constexpr double I8_FULL = 2139062142.0;              // 0x7F7F7F7E: four digits of 127, less one for the rounding
constexpr double I8_INV_FULL = 1.0 / 2139062142.0;
__device__ __forceinline__ bool i8_nonfinite(unsigned mbits) { return mbits >= 0x7f800000u; }
// scale with rint(m * scale) <= I8_FULL + 1; an all-zero block takes any scale
__device__ __forceinline__ double i8_scale(unsigned mbits) {
  return mbits ? I8_FULL / (double)__uint_as_float(mbits) : 1.0;
}
// 1 / scale to three roundings (the product scale * inverse differs from 1 by 3 * 2^-53 at most); NaN for Inf/NaN
__device__ __forceinline__ double i8_inverse_scale(unsigned mbits) {
  return i8_nonfinite(mbits) ? __longlong_as_double(0x7ff8000000000000ll) : (double)__uint_as_float(mbits) * I8_INV_FULL;
}

// rint(x * scale) as the low word of x * scale + 1.5 * 2^52 in fp64 (one fused operation: exact product, one
// rounding to nearest even), for |x * scale| < 2^31.  An even integer `plus` < 2^31 added to the constant comes out
// added to the result (mod 2^32) for free: the sum is still an integer plus the product, and ties still go to the
// even neighbour.
template <int plus = 0>
__device__ __forceinline__ int i8_fixed(float x, double scale) {
  static_assert(plus >= 0 && plus % 2 == 0, "an even offset keeps round-to-nearest-even on the product");
  return __double2loint(__builtin_fma((double)x, scale, 6755399441055744.0 + (double)plus));
}

__device__ __forceinline__ int i8_max3(int a, int b, int c) {
  int d;
  asm("v_max3_i32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}
__device__ __forceinline__ unsigned i8_max3(unsigned a, unsigned b, unsigned c) {
  unsigned d;
  asm("v_max3_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

// 4 x 4 byte transpose: x[c] holds the 4 digits of channel c; y[k] receives digit k of the 4 channels.
__device__ __forceinline__ void i8_transpose4(const int (&x)[4], int (&y)[4]) {
  const unsigned lo01 = __builtin_amdgcn_perm(x[1], x[0], 0x05010400u);  // x0.0 x1.0 x0.1 x1.1
  const unsigned hi01 = __builtin_amdgcn_perm(x[1], x[0], 0x07030602u);  // x0.2 x1.2 x0.3 x1.3
  const unsigned lo23 = __builtin_amdgcn_perm(x[3], x[2], 0x05010400u);
  const unsigned hi23 = __builtin_amdgcn_perm(x[3], x[2], 0x07030602u);
  y[0] = (int)__builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
  y[1] = (int)__builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
  y[2] = (int)__builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
  y[3] = (int)__builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
}

// Maximum over the wavefront, returned in every lane: four cross-lane steps inside each row of 16 lanes (data
// parallel primitives: no LDS round trips), then the four rows through scalar registers.
__device__ __forceinline__ unsigned i8_wave_max(unsigned m) {
  int v = (int)m;  // bit patterns with the sign cleared: signed and unsigned order agree
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, false));  // row_mirror
  const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
  const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
  return (unsigned)max(max(r0, r1), max(r2, r3));
}

// Minimum over the wavefront of bit patterns with the sign cleared, returned in every lane.
__device__ __forceinline__ unsigned i8_wave_min(unsigned m) {
  int v = (int)m;
  v = min(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));
  v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));
  v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));
  v = min(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, false));
  const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
  const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
  return (unsigned)min(min(r0, r1), min(r2, r3));
}

__device__ __forceinline__ i4 mfma_i8(i4 a, i4 b, i4 c) { return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0); }

// MIND: the lowest digit diagonal k + l that is kept: 3 (10 products, the default) or 2 (13 products).
template <int W, int ROWS, int MIND = 3>
__global__ __launch_bounds__(WG_THREADS, 2) void gconv_i8_kernel(GconvI8Args p) {
  static_assert(MIND == 2 || MIND == 3, "10 or 13 digit products");
  using Gm = GconvI8Geom<W, ROWS>;
  constexpr int C = Gm::C, F = Gm::F, KH = Gm::KH, KW = Gm::KW, OW = Gm::OW, PLANE = Gm::PLANE, BUF = Gm::BUF,
                NFC = Gm::NFC, NHALF = Gm::NHALF;
  constexpr int WN = F * C * KH * KW, WPT = WN / WG_THREADS;  // filter bank of a group; floats per thread
  static_assert(WN % WG_THREADS == 0, "whole filter-bank floats per thread");
  extern __shared__ __attribute__((aligned(16))) char gi8_lds[];
  unsigned* maxw = reinterpret_cast<unsigned*>(gi8_lds + Gm::MISC);     // [2][4] band maxima per wavefront
  unsigned* minw = maxw + 8;                                            // [2][4] smallest per-thread maximum per wavefront

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int kwq = q < KW ? q : KW - 1;  // slot group 3 is padding: it re-reads kw = 2 against zero weights
  const int H = p.H, OH = H - KH + 1;
  const int npix = OH * OW;
  const int nbands = OH / ROWS;
  const int plane = H * W;
  // ---- this workgroup's run of bands [u, u1) in the order (g, n, band)
  int u, u1;
  {
    // 32-bit arithmetic: the host checks bands * (workgroups + 1) < 2^31
    const unsigned tb = (unsigned)(p.N * p.G * nbands);
    const unsigned w = blockIdx.x;
    if (p.halves) {
      const unsigned hv = (unsigned)p.halves, pr = w % hv;
      const unsigned s0 = tb * pr / hv, e0 = tb * (pr + 1) / hv;
      const unsigned mid = s0 + (e0 - s0) * (unsigned)p.num / (unsigned)p.den;
      u = (int)(w < hv ? s0 : mid);
      u1 = (int)(w < hv ? mid : e0);
    } else {
      u = (int)(tb * w / gridDim.x);
      u1 = (int)(tb * (w + 1) / gridDim.x);
    }
  }
  if (u >= u1) return;
  // band number -> group, image, band of the image
  int g, b, img;
  auto decode = [&](int unit) {
    const int pair = unit / nbands;
    b = unit - pair * nbands;
    g = pair / p.N;
    img = (pair - g * p.N) * p.G + g;  // n*G + g
  };

  // ---- the band being fetched: two units and (first NHALF threads) one half unit per thread
  const bool has_half = wave * WAVE < NHALF;  // whole wavefronts only
  const int hunit = 2 * WG_THREADS + min(tid, NHALF - 1) / 2, hhalf = tid & 1;
  f4 pre[2][4];   // [round][channel of the group], 4 pixels each
  f2 preh[4];
  const char* fimg;   // image block the band is fetched from
  unsigned foff;      // byte offset of the band inside a channel plane
  auto set_fetch = [&](int im, int b) {
    fimg = reinterpret_cast<const char*>(p.I + (int64_t)im * C * plane);
    foff = 4u * (unsigned)(b * ROWS * W);
  };
  // piece 0, 1: the two units; piece 2: the half unit.  Uniform base + 32-bit byte offset (the host checks 64*H*W < 2^32).
  auto fetch_piece = [&](auto pc_c) {
    constexpr int pc = decltype(pc_c)::value;
    if constexpr (pc < 2) {
      const int unit = tid + pc * WG_THREADS, cg = unit & 3, px4 = unit >> 2;
      const unsigned off = foff + 4u * (unsigned)((4 * cg) * plane + 4 * px4);
#pragma unroll
      for (int c = 0; c < 4; c++) pre[pc][c] = *reinterpret_cast<const f4*>(fimg + (off + 4u * (unsigned)(c * plane)));
    } else if (has_half) {
      const int cg = hunit & 3, px4 = hunit >> 2;
      const unsigned off = foff + 4u * (unsigned)((4 * cg) * plane + 4 * px4 + 2 * hhalf);
#pragma unroll
      for (int c = 0; c < 4; c++) preh[c] = *reinterpret_cast<const f2*>(fimg + (off + 4u * (unsigned)(c * plane)));
    }
  };
  using std::integral_constant;
  decode(u);
  // The first filter bank is requested before the first band: loads return in order, and at the start of the
  // launch every workgroup's band fetch (20 MB over the chip) would otherwise stand between a workgroup and the
  // 9 KB it needs before anything else can begin.
  float wpre[WPT];
  {
    const float* wg = p.W1 + (int64_t)g * WN;
#pragma unroll
    for (int j = 0; j < WPT; j++) wpre[j] = wg[tid + j * WG_THREADS];
  }
  set_fetch(img, b);
  fetch_piece(integral_constant<int, 0>{});
  fetch_piece(integral_constant<int, 1>{});
  fetch_piece(integral_constant<int, 2>{});

  i4 a[KH][4];     // a[kh][k]: digit k of W1[g][r16][c = byte][kh][kw = q], zeros for q = 3
  double fa[4];    // 2^24 / scale of filter row 4q + v (NaN if the row holds Inf/NaN)
  float bz[4];     // bias of filter row 4q + v
  float wspread = 0.f;  // largest max|w| / mean|w| among the group's filter rows (uniform)
  int it = 0;      // bands staged so far by this workgroup: LDS buffer parity
  int g_bank = -1; // group whose filter bank the A operands hold
  for (; u < u1; u++, it++) {
    decode(u);
    char* dst = reinterpret_cast<char*>(p.O + (int64_t)img * F * npix);
    // ---- filter bank -> A operands, through the band buffer that is staged next (free: it was last read two bands ago).
    // Every lane needs digit records of all 16 channels of its (filter row, kw) for the 3 kh; wavefront w slices
    // channels 4w..4w+3 and the four share their dwords through LDS: record (kh, k) of a lane at
    // arec + ((kh*4 + k)*64 + lane)*16, dword w.
    if (g != g_bank) {
      if (g_bank >= 0) {  // a later bank of the run (the first one is already on its way)
        const float* wg = p.W1 + (int64_t)g * WN;
#pragma unroll
        for (int j = 0; j < WPT; j++) wpre[j] = wg[tid + j * WG_THREADS];
      }
      g_bank = g;
      __syncthreads();  // slower wavefronts may still be reading their output staging in this buffer
      float* wl = reinterpret_cast<float*>(gi8_lds + (it & 1) * BUF);
      char* arec = reinterpret_cast<char*>(wl) + 16384;
      static_assert(WN * 4 <= 16384 && 16384 + KH * 4 * WAVE * 16 <= BUF, "scratch must fit one band buffer");
      // filter rows are WROW floats apart (odd): the 16 rows that the lanes of a read address fall into 16 banks
      constexpr int WROW = C * KH * KW + 1;
      static_assert(F * WROW * 4 <= 16384, "padded filter bank must end before the digit records");
#pragma unroll
      for (int j = 0; j < WPT; j++) {
        const int i = tid + j * WG_THREADS, f = i / (C * KH * KW);
        wl[i + f] = wpre[j];
      }
      __syncthreads();
      const float* wp = wl + r16 * WROW + kwq;
      unsigned m = 0;
#pragma unroll
      for (int kh = 0; kh < KH; kh++)
#pragma unroll
        for (int c = 0; c < C; c++) m = max(m, __float_as_uint(wp[c * (KH * KW) + kh * KW]) & 0x7fffffffu);
      m = max(m, (unsigned)__shfl_xor((int)m, 16));
      m = max(m, (unsigned)__shfl_xor((int)m, 32));
      const double sa = i8_scale(m);  // m = max|w| over the filter row
      {
        // max / mean of the row's 144 magnitudes (lanes q = 0..2 hold one kw each; q = 3 re-reads kw = 2: left out),
        // then the largest of the 16 rows
        float sum = 0.f;
#pragma unroll
        for (int kh = 0; kh < KH; kh++)
#pragma unroll
          for (int c = 0; c < C; c++) sum += __builtin_fabsf(wp[c * (KH * KW) + kh * KW]);
        sum = q < KW ? sum : 0.f;
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        const float ratio = sum > 0.f ? __uint_as_float(m) * (float)(C * KH * KW) / sum : 1.f;  // an all-zero row: 1
        wspread = __uint_as_float(i8_wave_max(__float_as_uint(ratio)));  // ratio >= 1 > 0: bit patterns order like values
      }
#pragma unroll
      for (int kh = 0; kh < KH; kh++) {
        int d[4], y[4];
#pragma unroll
        for (int c = 0; c < 4; c++)
          d[c] = i8_fixed<0x00808080>(wp[(4 * wave + c) * (KH * KW) + kh * KW], sa) ^ 0x00808080;  // byte k = digit k
        i8_transpose4(d, y);
#pragma unroll
        for (int k = 0; k < 4; k++)
          *reinterpret_cast<int*>(arec + ((kh * 4 + k) * WAVE + lane) * 16 + 4 * wave) = q < KW ? y[k] : 0;
      }
      __syncthreads();
#pragma unroll
      for (int kh = 0; kh < KH; kh++)
#pragma unroll
        for (int k = 0; k < 4; k++) a[kh][k] = *reinterpret_cast<const i4*>(arec + ((kh * 4 + k) * WAVE + lane) * 16);
#pragma unroll
      for (int v = 0; v < 4; v++) {
        fa[v] = 16777216.0 * i8_inverse_scale((unsigned)__shfl((int)m, 4 * q + v));  // lane 4q+v holds filter row 4q+v
        bz[v] = p.bias ? p.bias[g * F + 4 * q + v] : 0.f;
      }
      // the staging below overwrites this scratch only after the next barrier, which every wavefront reaches after these reads
    }

    {
      char* buf = gi8_lds + (it & 1) * BUF;
      // ---- largest magnitude of the band: bit patterns order like magnitudes.  Positive values (and NaNs) win a
      // signed maximum, negative ones an unsigned maximum: one instruction per two elements each.
      int mp = 0;
      unsigned mn = 0;
      auto take = [&](float x, float y) {
        mp = i8_max3(mp, __float_as_int(x), __float_as_int(y));
        mn = i8_max3(mn, __float_as_uint(x), __float_as_uint(y));
      };
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int c = 0; c < 4; c++) {
          take(pre[j][c][0], pre[j][c][1]);
          take(pre[j][c][2], pre[j][c][3]);
        }
      if (has_half) {
#pragma unroll
        for (int c = 0; c < 4; c++) take(preh[c][0], preh[c][1]);
      }
      unsigned m = max((unsigned)mp, mn & 0x7fffffffu);
      const unsigned tmin = i8_wave_min(m);  // smallest per-thread maximum of this wavefront
      m = i8_wave_max(m);
      if (lane == 0) {
        maxw[(it & 1) * 4 + wave] = m;
        minw[(it & 1) * 4 + wave] = tmin;
      }
      __syncthreads();
      m = max(max(maxw[(it & 1) * 4 + 0], maxw[(it & 1) * 4 + 1]), max(maxw[(it & 1) * 4 + 2], maxw[(it & 1) * 4 + 3]));
      m = (unsigned)__builtin_amdgcn_readfirstlane((int)m);  // max|x| over the band
      // heavy-tailed band?  S = (band maximum / smallest per-thread maximum) * (spread of the filter rows); a thread
      // that saw only zeros makes S infinite.  Uniform over the workgroup.
      bool heavy = p.force13 > 0;
      if (MIND == 3 && p.force13 == 0) {
        unsigned t = min(min(minw[(it & 1) * 4 + 0], minw[(it & 1) * 4 + 1]), min(minw[(it & 1) * 4 + 2], minw[(it & 1) * 4 + 3]));
        t = (unsigned)__builtin_amdgcn_readfirstlane((int)t);
        heavy = !(__uint_as_float(m) * wspread <= I8_HEAVY_STAT * __uint_as_float(t));  // (NaN compares false: heavy)
      }

      // ---- slice and stage: digit plane k, record of pixel pi at byte k*PLANE + 16*pi, channels 4cg.. at +4cg
      {
        const double sv = i8_scale(m);  // the same in every lane: kept in scalar registers
        const double scale = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(sv)),
                                              __builtin_amdgcn_readfirstlane(__double2loint(sv)));
        auto put = [&](float x0, float x1, float x2, float x3, int cg, int pixel) {  // 4 channels of one pixel
          // v + 0x00808080 (added inside the rounding) makes byte k digit k plus 128; flipping bit 7 of bytes 0..2 afterwards gives the digits,
          // and that flip commutes with the byte transpose: three instructions per four elements instead of four
          int d[4] = {i8_fixed<0x00808080>(x0, scale), i8_fixed<0x00808080>(x1, scale),
                      i8_fixed<0x00808080>(x2, scale), i8_fixed<0x00808080>(x3, scale)}, y[4];
          i8_transpose4(d, y);
#pragma unroll
          for (int k = 0; k < 4; k++)
            *reinterpret_cast<int*>(buf + k * PLANE + 16 * pixel + 4 * cg) = k < 3 ? y[k] ^ (int)0x80808080 : y[k];
        };
#pragma unroll
        for (int j = 0; j < 2; j++) {
          const int unit = tid + j * WG_THREADS, cg = unit & 3, px4 = unit >> 2;
#pragma unroll
          for (int e = 0; e < 4; e++) put(pre[j][0][e], pre[j][1][e], pre[j][2][e], pre[j][3][e], cg, 4 * px4 + e);
        }
        if (has_half) {
          const int cg = hunit & 3, px4 = hunit >> 2;
          if (tid < NHALF) {
#pragma unroll
            for (int e = 0; e < 2; e++) put(preh[0][e], preh[1][e], preh[2][e], preh[3][e], cg, 4 * px4 + 2 * hhalf + e);
          }
        }
      }
      __syncthreads();

      // ---- what to fetch while this band is contracted: the next band of the run
      const bool more = u + 1 < u1;
      const int b_now = b;
      if (more) {
        decode(u + 1);
        set_fetch(img, b);
      }
      // what one unit of the combined diagonals is worth, per filter row of this lane; NaN if the band or the row
      // holds Inf/NaN
      const double invb = i8_inverse_scale(m);
      double fo[4];
#pragma unroll
      for (int v = 0; v < 4; v++) fo[v] = fa[v] * invb;

      const int h0 = b_now * ROWS + 2 * wave;  // first output row of this wavefront in this band
      // Outputs are staged per wavefront in the idle band buffer as [filter][2 rows][OW] and written out after the
      // sweeps with 16-byte stores, a filter's two rows (2*OW*4 contiguous bytes of O) at a time: 4-byte stores of
      // 64-byte pieces of four different rows keep the path to HBM busy four times as long.
      char* ostage = gi8_lds + ((it + 1) & 1) * BUF + wave * Gm::OSTAGE;
      char* olane = ostage + (4 * q) * (Gm::OSF * 4) + r16 * 4;
      // One sweep: NR output rows per lane, NR + 2 input rows starting at the lane's LDS pointer `base`
      // (input row of its first output row, column of its pixel + kw).  orow/ocol: the lane's first output
      // row and its column.  PIECE: the fetch piece of the next band to issue during this sweep, or -1.
      // FIX: the second, lighter kind of sweep: only the diagonal k + l = 2, added to what the first kind staged.
      auto sweep = [&](auto nr_c, auto piece_c, auto col_c, auto fix_c, const char* base, char* obase) {
        constexpr int NR = decltype(nr_c)::value, PIECE = decltype(piece_c)::value, COL = decltype(col_c)::value;
        constexpr bool FIX = decltype(fix_c)::value;
        constexpr int ND = FIX ? 1 : 7 - MIND;
        constexpr int NL = FIX ? 3 : 4;  // digit planes of the input that the sweep reads
        i4 acc[NR][ND];  // diagonals k + l = MIND .. 6
#pragma unroll
        for (int hl = 0; hl < NR; hl++)
#pragma unroll
          for (int d = 0; d < ND; d++) acc[hl][d] = i4{0, 0, 0, 0};
        i4 bc[4], bn[4];
#pragma unroll
        for (int l = 0; l < NL; l++) bc[l] = *reinterpret_cast<const i4*>(base + l * PLANE);
        auto row = [&](auto r_c) {
          constexpr int r = decltype(r_c)::value;
          if constexpr (r + 1 < NR + 2) {
#pragma unroll
            for (int l = 0; l < NL; l++) bn[l] = *reinterpret_cast<const i4*>(base + l * PLANE + (r + 1) * W * 16);
          }
          if constexpr (PIECE >= 0 && r == 1) {
            if (more) fetch_piece(integral_constant<int, PIECE >= 0 ? PIECE : 0>{});
          }
          // pin "reads of row r+1, then MFMAs of row r"
          __builtin_amdgcn_sched_barrier(0);
          // digit pairs (k of the weights, l of the input), ordered so that consecutive MFMAs hit different diagonals
          constexpr int NP = MIND == 3 ? 10 : 13;  // the last three pairs are the diagonal k + l = 2
          constexpr int PK[13] = {3, 3, 3, 3, 2, 2, 2, 1, 1, 0, 2, 1, 0};
          constexpr int PL[13] = {3, 2, 1, 0, 3, 2, 1, 3, 2, 3, 0, 1, 2};
#pragma unroll
          for (int i = FIX ? 10 : 0; i < (FIX ? 13 : NP); i++)
#pragma unroll
            for (int hl = 0; hl < NR; hl++) {
              const int kh = r - hl;
              constexpr int D0 = FIX ? 2 : MIND;
              if (kh >= 0 && kh < KH)
                acc[hl][PK[i] + PL[i] - D0] = mfma_i8(a[kh][PK[i]], bc[PL[i]], acc[hl][PK[i] + PL[i] - D0]);
            }
#pragma unroll
          for (int l = 0; l < NL; l++) bc[l] = bn[l];
          __builtin_amdgcn_sched_barrier(0);
        };
        row(integral_constant<int, 0>{});
        row(integral_constant<int, 1>{});
        row(integral_constant<int, 2>{});
        if constexpr (NR == 2) row(integral_constant<int, 3>{});
        static_assert(NR == 1 || NR == 2, "one or two output rows per sweep");
        if constexpr (FIX) {
          // the diagonal k + l = 2 is worth 1/256 of a unit of the combined diagonals; it joins the staged value (this
          // lane wrote it, this lane reads it) in fp64, and the sum is rounded to fp32 again
#pragma unroll
          for (int hl = 0; hl < NR; hl++)
#pragma unroll
            for (int v = 0; v < 4; v++) {
              float* o = reinterpret_cast<float*>(obase + (v * Gm::OSF + hl * OW + COL) * 4);
              *o = (float)__builtin_fma((double)acc[hl][0][v] * 0.00390625, fo[v], (double)*o);
            }
          return;
        }
        // ---- exact recombination of the diagonals, scaling, bias, single rounding
#pragma unroll
        for (int hl = 0; hl < NR; hl++) {
#pragma unroll
          for (int v = 0; v < 4; v++) {
            // |P_6| <= 144 * 2^14, |P_5| <= 2 * 144 * 2^14, |P_4| <= 3 * 144 * 2^14, |P_3| <= 4 * 144 * 2^14
            const int hi = acc[hl][ND - 1][v] * 256 + acc[hl][ND - 2][v];  // |.| < 2^30
            const int lo = acc[hl][ND - 3][v] * 256 + acc[hl][ND - 4][v];  // |.| < 2^31
            double rr = __builtin_fma((double)hi, 65536.0, (double)lo);  // sum_d P_d 256^(d-3), exact
            if constexpr (MIND == 2) rr = __builtin_fma((double)acc[hl][0][v], 0.00390625, rr);
            *reinterpret_cast<float*>(obase + (v * Gm::OSF + hl * OW + COL) * 4) =
                (float)__builtin_fma(rr, fo[v], (double)bz[v]);
          }
        }
      };
      const char* lbase = buf + ((2 * wave) * W + r16 + kwq) * 16;
      using std::false_type;
      using std::true_type;
      sweep(integral_constant<int, 2>{}, integral_constant<int, 0>{}, integral_constant<int, 0>{}, false_type{}, lbase, olane);
      sweep(integral_constant<int, 2>{}, integral_constant<int, 1>{}, integral_constant<int, 16>{}, false_type{}, lbase + 256, olane);
      sweep(integral_constant<int, 2>{}, integral_constant<int, 2>{}, integral_constant<int, 32>{}, false_type{}, lbase + 512, olane);
      static_assert(NFC == 3, "three full columns are written out above");
      // last 8 columns of both rows in one tile: lanes 0-7 row h0, lanes 8-15 row h0 + 1
      const int hr = r16 >> 3;
      const char* lbase8 = buf + ((2 * wave + hr) * W + 16 * NFC + (r16 & 7) + kwq) * 16;
      char* olane8 = olane + (hr * OW + (r16 & 7) - r16) * 4;
      sweep(integral_constant<int, 1>{}, integral_constant<int, -1>{}, integral_constant<int, 16 * NFC>{}, false_type{}, lbase8, olane8);
      if constexpr (MIND == 3) {
        if (heavy) {  // uniform over the workgroup: the same sweeps again for the diagonal k + l = 2
          sweep(integral_constant<int, 2>{}, integral_constant<int, -1>{}, integral_constant<int, 0>{}, true_type{}, lbase, olane);
          sweep(integral_constant<int, 2>{}, integral_constant<int, -1>{}, integral_constant<int, 16>{}, true_type{}, lbase + 256, olane);
          sweep(integral_constant<int, 2>{}, integral_constant<int, -1>{}, integral_constant<int, 32>{}, true_type{}, lbase + 512, olane);
          sweep(integral_constant<int, 1>{}, integral_constant<int, -1>{}, integral_constant<int, 16 * NFC>{}, true_type{}, lbase8, olane8);
        }
      }
      // ---- staged outputs -> O: instruction j writes filters 2j (lanes 0-31) and 2j+1 (lanes 32-63), 16 bytes per
      // lane; the staging is private to the wavefront, so its own LDS writes only have to have landed
      {
        constexpr int PIECES = 2 * OW * 4 / 16;  // 16-byte pieces of a filter's two rows
        const int pc = lane & 31, fsel = lane >> 5;
        const char* srd = ostage + fsel * (Gm::OSF * 4) + pc * 16;
        char* gwr = dst + 4 * (fsel * npix + h0 * OW) + pc * 16;
        if (pc < PIECES) {
#pragma unroll
          for (int j = 0; j < 8; j++) {
            const f4 v = *reinterpret_cast<const f4*>(srd + j * 2 * Gm::OSF * 4);
            // written once, never read again by this kernel: a streaming store keeps the output out of the way of
            // the input rows that the next band re-reads from L2 (measured: 10 % of the launch)
            store_stream(reinterpret_cast<f4*>(gwr + (int64_t)j * 2 * npix * 4), v);
          }
        }
      }
    }
  }
}

}  // namespace tc355
