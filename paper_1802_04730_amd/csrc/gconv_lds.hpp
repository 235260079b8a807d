// Tuned grouped convolution (Section 7, listing gconv) for channel counts that
// fit the matrix core exactly: C % 4 == 0 input channels and F % 16 == 0 output
// channels per group, small filters.
//
// Mapping (one workgroup = 4 wavefronts):
//   workgroup  -> one (image n, group g) and a block of 64*TP consecutive
//                 output pixels (pixels are numbered h*OW + w, so a block is a
//                 band of output rows);
//   LDS        -> the band of input rows those pixels touch, all C channels,
//                 fp32, plane stride PS chosen = 16 (mod 64) words so that the
//                 four k slots of a wavefront read disjoint banks;
//                 The filter bank of the group sits behind it, fp32, already
//                 permuted into MFMA A-operand order (one word per lane and
//                 step), so it costs no registers;
//   registers  -> TP accumulator tiles per wavefront.
// The reduction is consumed in the order (kh, kw, c/4) with k slot q carrying
// channel 4*(c/4)+q, so that every LDS read of a step is "lane base + constant".
// Each 16x16x4 fp64 MFMA needs one 4-byte LDS read and one widening, far below
// what LDS and the vector ALU can deliver, so the kernel is bound by the fp64
// matrix pipe.  The bias is added in fp64 before the single rounding to fp32.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct GconvLdsArgs {
  const float* I;
  const float* W1;
  const float* bias;  // or nullptr
  float* O;
  int G, H, W, OH, OW;
  int PS;       // LDS plane stride in floats
  int pblocks;  // pixel blocks per (n,g)
  int64_t ngs;  // N*G
};

// Plane stride: at least `len` floats, congruent to 16 modulo 64, multiple of 4.
inline int gconv_plane_stride(int len) {
  int ps = (len + 3) & ~3;
  while ((ps & 63) != 16) ps += 4;
  return ps;
}

// Rows of input a block of `pixels` consecutive output pixels can touch.
inline int gconv_band_rows(int pixels, int OW, int KH) {
  const int out_rows = (pixels % OW == 0) ? pixels / OW : pixels / OW + 2;
  return out_rows + KH - 1;
}

template <int C, int F, int KH, int KW, int TP>
__global__ __launch_bounds__(WG_THREADS, 3) void gconv_lds_kernel(GconvLdsArgs p) {
  static_assert(C % 4 == 0 && F % 16 == 0, "channel counts must fit the 16x16x4 tile");
  constexpr int NS = KH * KW * (C / 4);  // MFMA steps per output tile
  constexpr int FT = F / 16;
  extern __shared__ float lds[];

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1), wave = tid / WAVE;
  const int r16 = lane & 15, q = lane >> 4;

  // Consecutive workgroup ids are dealt round-robin to the 8 XCDs; give each XCD
  // a contiguous range of blocks so neighbouring bands share an L2.
  const int64_t nblocks = (int64_t)gridDim.x;
  int64_t blk = blockIdx.x;
  if ((nblocks & 7) == 0) blk = (blk & 7) * (nblocks >> 3) + (blk >> 3);
  const int pb = (int)(blk % p.pblocks);
  const int64_t ng = blk / p.pblocks;
  const int g = (int)(ng % p.G);

  const int H = p.H, W = p.W, OW = p.OW, PS = p.PS;
  const int npix = p.OH * OW;
  const int P0 = pb * (64 * TP);
  const int h_first = P0 / OW;
  const int plast = min(P0 + 64 * TP, npix) - 1;
  const int rows = plast / OW - h_first + KH;

  // ---- filter bank of this group -> LDS, already in MFMA A-operand order:
  //      wl[(ft*NS + s)*64 + lane] = W1[g][ft*16 + r16][4*c4 + q][kh][kw],  s = (kh*KW + kw)*(C/4) + c4
  float* wl = lds + C * PS;
  for (int idx = tid; idx < FT * NS * WAVE; idx += WG_THREADS) {
    const int ln = idx & (WAVE - 1), fs = idx / WAVE;
    const int ft = fs / NS, st = fs - ft * NS;
    const int c4 = st % (C / 4), kk = st / (C / 4);  // kk = kh*KW + kw
    const int f = ft * 16 + (ln & 15), c = 4 * c4 + (ln >> 4);
    wl[idx] = p.W1[((int64_t)(g * F + f) * C + c) * (KH * KW) + kk];
  }

  // ---- input band -> LDS
  const float* src = p.I + ng * (int64_t)C * H * W + (int64_t)h_first * W;
  const int len = rows * W;
  const bool vec_ok = ((len & 3) == 0) && ((((int64_t)H * W) & 3) == 0) && (((h_first * W) & 3) == 0);
  if (vec_ok) {
    const int len4 = len >> 2;
    for (int idx = tid; idx < C * len4; idx += WG_THREADS) {
      const int c = idx / len4, i = idx - c * len4;
      const f4 v = *reinterpret_cast<const f4*>(src + (int64_t)c * H * W + 4 * i);
      *reinterpret_cast<f4*>(lds + c * PS + 4 * i) = v;
    }
  } else {
    for (int idx = tid; idx < C * len; idx += WG_THREADS) {
      const int c = idx / len, i = idx - c * len;
      lds[c * PS + i] = src[(int64_t)c * H * W + i];
    }
  }
  __syncthreads();

  // ---- contraction: this wavefront owns TP consecutive pixel tiles of the block
  int base[TP];
#pragma unroll
  for (int t = 0; t < TP; t++) {
    const int px = min(P0 + (wave * TP + t) * 16 + r16, npix - 1);
    const int h = px / OW;
    base[t] = q * PS + (h - h_first) * W + (px - h * OW);
  }
  d4 acc[FT][TP];
#pragma unroll
  for (int ft = 0; ft < FT; ft++)
#pragma unroll
    for (int t = 0; t < TP; t++) acc[ft][t] = d4_zero();

#pragma unroll
  for (int kh = 0; kh < KH; kh++)
#pragma unroll
    for (int kw = 0; kw < KW; kw++)
#pragma unroll
      for (int c4 = 0; c4 < C / 4; c4++) {
        const int s = (kh * KW + kw) * (C / 4) + c4;
        const int off = 4 * c4 * PS + kh * W + kw;
        double a[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ft++) a[ft] = (double)wl[(ft * NS + s) * WAVE + lane];
#pragma unroll
        for (int t = 0; t < TP; t++) {
          const double b = (double)lds[base[t] + off];
#pragma unroll
          for (int ft = 0; ft < FT; ft++) acc[ft][t] = mfma_f64(a[ft], b, acc[ft][t]);
        }
      }

  // ---- epilogue: bias in fp64, one rounding, 64-byte row segments
  float* op = p.O + ng * (int64_t)F * npix;
#pragma unroll
  for (int ft = 0; ft < FT; ft++)
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const int f = ft * 16 + d_row(q, v);
      const double bz = p.bias ? (double)p.bias[g * F + f] : 0.0;
#pragma unroll
      for (int t = 0; t < TP; t++) {
        const int px = P0 + (wave * TP + t) * 16 + r16;
        if (px < npix) op[(int64_t)f * npix + px] = (float)(acc[ft][t][v] + bz);
      }
    }
}

}  // namespace tc355
