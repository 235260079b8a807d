// Grouped convolution (Section 7, listing gconv) for FEW channels per group
// (C and F multiples of 4, up to 8; the paper's table shapes (4,4,56,56) and
// (8,8,28,28), and the same with a border of one pixel: widths 58 and 30), image width known at compile time:
//
//   O(n,g,o,h,w) = sum_{i,kh,kw} I(n,g,i,h+kh,w+kw) * W1(g,o,i,kh,kw) + bias(g*F+o)
//
// With 4 or 8 filters a 16 x 16 MFMA tile would be three quarters or half
// padding.  v_mfma_f64_4x4x4_4b_f64 multiplies four independent 4 x 4 x 4 blocks
// per instruction at the same flop rate; measured layout (one-hot probe), lane =
// 16*k + 4*blk + idx:
//   A: lane supplies A_blk[i = idx][k]      B: lane supplies B_blk[k][j = idx]
//   D: lane 16*i + 4*blk + j holds D_blk[i][j]
// Here all four blocks share A = the weights of 4 filters x 4 channels for one
// filter tap, and take 4 different pixel quads: one instruction contracts 4
// channels of one tap for 4 filters x 16 pixels, with no padding.  In the
// terms of the 16-wide kernels (r16 = lane % 16, q = lane / 16) the B operand
// is again I[channel 4*c4 + q][pixel r16], one 8-byte LDS read at a
// compile-time immediate; the A operand is W1[filter 4*fq + lane % 4][channel
// 4*c4 + q]; and the lane ends up with O[filter 4*fq + q][pixel r16].
//
// One workgroup per (image, group); bands of ROWS output rows; the band is
// widened to fp64 once and staged in LDS ([channel][pixels], plane stride
// = 16 mod 32 doubles); the filter bank sits in registers; the tiles of a band
// are dealt to the four wavefronts round-robin and advance TN at a time with the
// LDS reads one step ahead of the MFMAs.  Several workgroups per compute unit
// cover each other's staging.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct GconvQuadArgs {
  const float* I;
  const float* W1;
  const float* bias;  // or nullptr
  float* O;
  int G, H;
};

template <int C, int F, int KH, int KW, int W, int ROWS>
struct GconvQuadGeom {
  static constexpr int OW = W - KW + 1;
  static constexpr int IN_ROWS = ROWS + KH - 1;
  static constexpr int LEN = IN_ROWS * W;                          // floats per channel plane of a band
  static constexpr int PS = ((LEN + 31 - 16) / 32) * 32 + 16;      // plane stride in doubles, = 16 (mod 32), >= LEN
  static constexpr int LDS_BYTES = C * PS * 8;
  static constexpr int TILES = (ROWS * OW + 15) / 16;              // 16-pixel tiles per band
  static constexpr int CQ = C / 4, FQ = F / 4;
  static constexpr int NS = KH * KW * CQ;                          // reduction steps per tile
  static_assert(C % 4 == 0 && F % 4 == 0 && C <= 8 && F <= 8, "4 or 8 channels and filters per group");
  static constexpr int VEC = W % 4 == 0 ? 4 : 2;                   // floats per staging load: rows start 16- or 8-byte aligned
  static_assert(W % 2 == 0, "8-byte loads at least: every row starts 8-byte aligned");
  static_assert(PS >= LEN, "plane stride too small");
  static_assert((4 * (CQ - 1) * PS + (KH - 1) * W + KW - 1) * 8 < 65536, "LDS immediates out of range");
  static_assert(F * C * KH * KW * 4 <= LDS_BYTES, "the filter bank is parked in the band area first");
};

template <int C, int F, int KH, int KW, int W, int ROWS, int MINW>
__global__ __launch_bounds__(WG_THREADS, MINW) void gconv_quad_kernel(GconvQuadArgs p) {
  using Gm = GconvQuadGeom<C, F, KH, KW, W, ROWS>;
  constexpr int OW = Gm::OW, PS = Gm::PS, NS = Gm::NS, LEN = Gm::LEN, CQ = Gm::CQ, FQ = Gm::FQ, TILES = Gm::TILES;
  extern __shared__ __attribute__((aligned(16))) double gq_band[];  // [C][PS]

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

  // ---- filter bank -> registers: a[s][fq] = W1[g][4*fq + lane%4][4*c4 + q][kh][kw], s = (kh*KW + kw)*CQ + c4.
  // The bank of a group is one contiguous block: fetch it with coalesced loads, park it in the (still unused)
  // band area, and let every lane pick its values.
  double a[NS][FQ];
  {
    constexpr int WN = F * C * KH * KW;
    float* wl = reinterpret_cast<float*>(gq_band);
    const float* wg = p.W1 + (int64_t)g * WN;
    for (int i = tid; i < WN; i += WG_THREADS) wl[i] = wg[i];
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KH * KW; kk++)
#pragma unroll
      for (int c4 = 0; c4 < CQ; c4++)
#pragma unroll
        for (int fq = 0; fq < FQ; fq++)
          a[kk * CQ + c4][fq] = (double)wl[((4 * fq + (lane & 3)) * C + 4 * c4 + q) * (KH * KW) + kk];
  }
  double bz[FQ];  // the lane's outputs belong to filter 4*fq + q
#pragma unroll
  for (int fq = 0; fq < FQ; fq++) bz[fq] = p.bias ? (double)p.bias[g * F + 4 * fq + q] : 0.0;

  for (int b = 0; b < nbands; b++) {
    __syncthreads();  // the previous band (or the parked filter bank) has been read by everyone
    // ---- stage the band: rows b*ROWS .. of every channel, widened to fp64; rows past the image are skipped.
    // W is a multiple of 4 (of 2), so planes, band starts and row ends are 16-byte (8-byte) aligned.  All loads are
    // issued before the first conversion (one at a time, every load would wait for the previous one's round trip).
    const int h0 = b * ROWS;
    const int avail = min((H - h0) * W, LEN);  // floats of each plane that belong to this band (a multiple of VEC)
    {
      constexpr int VEC = Gm::VEC, LENV = LEN / VEC, NLD = (C * LENV + WG_THREADS - 1) / WG_THREADS;
      static_assert(LEN % VEC == 0, "whole loads");
      Vec<float, VEC> v[NLD];
#pragma unroll
      for (int j = 0; j < NLD; j++) {
        const int u = min(tid + j * WG_THREADS, C * LENV - 1);
        const int c = u / LENV, i = min(VEC * (u - c * LENV), avail - VEC);  // clamped, never skipped per lane
        v[j] = load_vec<float, VEC>(src + c * plane + (int64_t)h0 * W + i);
      }
#pragma unroll
      for (int j = 0; j < NLD; j++) {
        const int u = tid + j * WG_THREADS;
        const int c = u / LENV, i = VEC * (u - c * LENV);
        if (u < C * LENV && i < avail) {
          double* d = gq_band + c * PS + i;  // PS and i are even: 16-byte aligned pairs
#pragma unroll
          for (int e = 0; e < VEC; e += 2) {
            const dbl2 pr = {(double)v[j].e[e], (double)v[j].e[e + 1]};
            *reinterpret_cast<dbl2*>(d + e) = pr;
          }
        }
      }
    }
    __syncthreads();

    const int P0 = b * ROWS * OW;
    const int band_px = min(ROWS * OW, npix - P0);  // output pixels of this band
    // tiles of the band are dealt round-robin: wavefront w takes tiles w, w+4, ...; TN of them advance together
    constexpr int TN = 4;
    for (int t0 = wave; t0 < TILES; t0 += WAVES_PER_WG * TN) {
      const double* bp[TN];
      double acc[TN][FQ], bcur[TN], bnxt[TN];
#pragma unroll
      for (int t = 0; t < TN; t++) {
        const int tile = t0 + t * WAVES_PER_WG;
        const int px = min(tile * 16 + r16, band_px - 1);  // clamped: a ragged tile recomputes the last pixel
        bp[t] = gq_band + q * PS + (px / OW) * W + (px % OW);
#pragma unroll
        for (int fq = 0; fq < FQ; fq++) acc[t][fq] = bz[fq];  // start from the bias: one add less per output
        bcur[t] = bp[t][0];
      }
#pragma unroll
      for (int s = 0; s < NS; s++) {
        if (s + 1 < NS) {
          const int kk = (s + 1) / CQ, c4 = (s + 1) % CQ;
          const int off = 4 * c4 * PS + (kk / KW) * W + (kk % KW);
#pragma unroll
          for (int t = 0; t < TN; t++) bnxt[t] = bp[t][off];
        }
        __builtin_amdgcn_sched_barrier(0);  // reads of step s+1, then the MFMAs of step s
#pragma unroll
        for (int t = 0; t < TN; t++)
#pragma unroll
          for (int fq = 0; fq < FQ; fq++) acc[t][fq] = __builtin_amdgcn_mfma_f64_4x4x4f64(a[s][fq], bcur[t], acc[t][fq], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < TN; t++) bcur[t] = bnxt[t];
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int t = 0; t < TN; t++) {
        const int pl = (t0 + t * WAVES_PER_WG) * 16 + r16;  // pixel within the band
        if (pl < band_px) {
#pragma unroll
          for (int fq = 0; fq < FQ; fq++) dst[(int64_t)(4 * fq + q) * npix + P0 + pl] = (float)acc[t][fq];
        }
      }
    }
  }
}

}  // namespace tc355
