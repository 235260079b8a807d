// Shape-generic grouped convolution (Section 7, listing gconv):
//   O(n,g,o,h,w) = sum_{i,kh,kw} I(n,g,i,h+kh,w+kw) * W1(g,o,i,kh,kw) + bias(g*F+o)
// as an implicit contraction per (n,g): the filter bank of group g is a
// row-major F x (C*KH*KW) matrix (the A operand), the B operand is gathered
// from the input on the fly.  One wavefront owns 16 output channels x 16*TP
// consecutive output pixels of one (n,g) and feeds the fp64 MFMA directly from
// global memory.  Any extents; the tuned path for C%4==0, F%16==0 lives in
// gconv_lds.hpp.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct GconvArgs {
  const float* I;     // [N][G][C][H][W]
  const float* W1;    // [G][F][C][KH][KW]
  const float* bias;  // [G*F] or nullptr
  float* O;           // [N][G][F][OH][OW]
  int N, G, C, F, H, W, KH, KW, OH, OW;
  int tiles_f;   // ceil(F / 16)
  int strips_p;  // ceil(OH*OW / (16*TP))
  int64_t jobs;  // N*G*tiles_f*strips_p
};

template <int TP>
__global__ __launch_bounds__(WG_THREADS) void gconv_wave_kernel(GconvArgs p) {
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const int r16 = lane & 15, q = lane >> 4;
  const int64_t job = (int64_t)blockIdx.x * WAVES_PER_WG + wave;
  if (job >= p.jobs) return;

  const int sp = (int)(job % p.strips_p);
  int64_t rest = job / p.strips_p;
  const int tf = (int)(rest % p.tiles_f);
  const int64_t ng = rest / p.tiles_f;  // n*G + g
  const int g = (int)(ng % p.G);
  const int F = p.F, C = p.C, H = p.H, W = p.W, KH = p.KH, KW = p.KW;
  const int npix = p.OH * p.OW;
  const int CKK = C * KH * KW;

  const int f0 = tf * 16, p0 = sp * 16 * TP;
  const int frow = min(f0 + r16, F - 1);
  const float* wp = p.W1 + ((int64_t)g * F + frow) * CKK;
  const float* ip = p.I + ng * (int64_t)C * H * W;

  int pixoff[TP];
#pragma unroll
  for (int t = 0; t < TP; t++) {
    const int px = min(p0 + 16 * t + r16, npix - 1);
    pixoff[t] = (px / p.OW) * W + (px % p.OW);
  }
  d4 acc[TP];
#pragma unroll
  for (int t = 0; t < TP; t++) acc[t] = d4_zero();

  // this lane's reduction element kk = k0 + q, decoded as (c, kh, kw)
  int kw = q % KW, kh = (q / KW) % KH, c = q / (KW * KH);
  for (int k0 = 0; k0 < CKK; k0 += 4) {
    const int kk = k0 + q;
    const bool in = kk < CKK;
    const double a = in ? (double)wp[in ? kk : 0] : 0.0;
    const int koff = in ? (c * H + kh) * W + kw : 0;
#pragma unroll
    for (int t = 0; t < TP; t++) {
      const double bb = in ? (double)ip[koff + pixoff[t]] : 0.0;
      acc[t] = mfma_f64(a, bb, acc[t]);
    }
    kw += 4;
    while (kw >= KW) { kw -= KW; kh++; }
    while (kh >= KH) { kh -= KH; c++; }
  }

  float* op = p.O + ng * (int64_t)F * npix;
#pragma unroll
  for (int v = 0; v < 4; v++) {
    const int f = f0 + d_row(q, v);
    if (f >= F) continue;
    const double bz = p.bias ? (double)p.bias[g * F + f] : 0.0;
#pragma unroll
    for (int t = 0; t < TP; t++) {
      const int px = p0 + 16 * t + r16;
      if (px < npix) op[(int64_t)f * npix + px] = (float)(acc[t][v] + bz);
    }
  }
}

}  // namespace tc355
