// Grouped convolution (Section 7, listing gconv) for MANY channels on TINY
// images (the paper's table shape (N,G,F,C,W,H) = (32,32,32,32,7,7): 25 output
// pixels per image, a filter bank of 36 KiB per group):
//
//   O(n,g,o,h,w) = sum_{i,kh,kw} I(n,g,i,h+kh,w+kw) * W1(g,o,i,kh,kw) + bias(g*F+o)
//
// Here the filter bank is the big operand and an image the small one, so the
// bank stays put: a workgroup owns one group and a run of images.  Its four
// wavefronts are (filter tile ft, pixel tile pt) = 2 x 2; a wavefront keeps the
// 16 filters x C x KH x KW weights of its filter tile in registers as fp64
// MFMA A operands for all its images, and contracts them with one pixel tile
// (16 of the up to 32 output pixels) of each image, which is staged in LDS
// widened to fp64 ([channel][pixel], double-buffered so that the next image is
// staged while this one is contracted).  Same MFMA conventions as the band
// kernel: k slot q carries channel 4*c4 + q, every B operand is one 8-byte LDS
// read at a compile-time immediate.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct GconvTinyArgs {
  const float* I;
  const float* W1;
  const float* bias;  // or nullptr
  float* O;
  int N, G;
  int chunk;    // images per workgroup
  int nchunks;  // ceil(N / chunk)
};

template <int C, int F, int KH, int KW, int H, int W>
struct GconvTinyGeom {
  static constexpr int OH = H - KH + 1, OW = W - KW + 1, NPIX = OH * OW;
  static constexpr int LEN = H * W;                                 // floats per channel plane
  static constexpr int PS = ((LEN + 31 - 16) / 32) * 32 + 16;       // plane stride in doubles, = 16 (mod 32), >= LEN
  static constexpr int IMG = C * PS;                                // doubles per staged image
  static constexpr int NS = KH * KW * (C / 4);                      // MFMA steps per tile
  static constexpr int WN = F * C * KH * KW;                        // floats of one group's filter bank
  static constexpr int LDS_BYTES = (2 * IMG * 8 > WN * 4) ? 2 * IMG * 8 : WN * 4;
  static constexpr int NLD = (C * LEN + WG_THREADS - 1) / WG_THREADS;  // floats per thread and image
  static_assert(F == 32 && C % 4 == 0, "two filter tiles of 16");
  static_assert(NPIX > 16 && NPIX <= 32, "two pixel tiles");
  static_assert(PS >= LEN, "plane stride too small");
  static_assert((4 * (C / 4 - 1) * PS + (KH - 1) * W + KW - 1) * 8 < 65536, "LDS immediates out of range");
};

template <int C, int F, int KH, int KW, int H, int W>
__global__ __launch_bounds__(WG_THREADS, 2) void gconv_tiny_kernel(GconvTinyArgs p) {
  using Gm = GconvTinyGeom<C, F, KH, KW, H, W>;
  constexpr int OW = Gm::OW, NPIX = Gm::NPIX, LEN = Gm::LEN, PS = Gm::PS, IMG = Gm::IMG, NS = Gm::NS, WN = Gm::WN,
                NLD = Gm::NLD;
  extern __shared__ __attribute__((aligned(16))) double gt_img[];  // [2][C][PS]; first the parked filter bank

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int ft = wave >> 1, pt = wave & 1;  // filter tile, pixel tile of this wavefront
  const int g = blockIdx.x / p.nchunks;
  const int n0 = (blockIdx.x % p.nchunks) * p.chunk;
  const int n1 = min(n0 + p.chunk, p.N);

  // ---- this thread's share of an image: element idx = tid + 256 j of the C*LEN floats (contiguous in memory)
  float pre[NLD];
  auto fetch = [&](int n) {
    const float* src = p.I + ((int64_t)n * p.G + g) * (C * LEN);
#pragma unroll
    for (int j = 0; j < NLD; j++) pre[j] = src[min(tid + j * WG_THREADS, C * LEN - 1)];  // clamped, never skipped per lane
  };
  auto stage = [&](double* img) {
#pragma unroll
    for (int j = 0; j < NLD; j++) {
      const int idx = tid + j * WG_THREADS;
      if (idx < C * LEN) {
        const int c = idx / LEN;
        img[c * PS + (idx - c * LEN)] = (double)pre[j];
      }
    }
  };
  fetch(n0);  // in flight while the filter bank is set up

  // ---- filter bank of the group -> registers: a[s] = W1[g][16*ft + r16][4*c4 + q][kh][kw], s = (kh*KW + kw)*(C/4) + c4
  double a[NS];
  {
    float* wl = reinterpret_cast<float*>(gt_img);
    const float* wg = p.W1 + (int64_t)g * WN;
    {  // all loads first, then the LDS writes (one at a time, every load would wait for the previous round trip)
      constexpr int WU = WN / 4 / WG_THREADS;
      static_assert(WN % (4 * WG_THREADS) == 0, "whole 16-byte units per thread");
      f4 wv[WU];
#pragma unroll
      for (int j = 0; j < WU; j++) wv[j] = *reinterpret_cast<const f4*>(wg + 4 * (tid + j * WG_THREADS));
#pragma unroll
      for (int j = 0; j < WU; j++) *reinterpret_cast<f4*>(wl + 4 * (tid + j * WG_THREADS)) = wv[j];
    }
    __syncthreads();
    const float* wp = wl + ((16 * ft + r16) * C + q) * (KH * KW);
#pragma unroll
    for (int kk = 0; kk < KH * KW; kk++)
#pragma unroll
      for (int c4 = 0; c4 < C / 4; c4++) a[kk * (C / 4) + c4] = (double)wp[4 * c4 * (KH * KW) + kk];
  }
  double bz[4];  // D element v of a lane belongs to filter 16*ft + 4v + q
#pragma unroll
  for (int v = 0; v < 4; v++) bz[v] = p.bias ? (double)p.bias[g * F + 16 * ft + d_row(q, v)] : 0.0;
  __syncthreads();  // everyone has picked its weights: the LDS area is free for images
  stage(gt_img);
  if (n0 + 1 < n1) fetch(n0 + 1);
  __syncthreads();

  // the lane's pixel of the tile (clamped: lanes past the image recompute the last pixel and do not store)
  const int px = min(16 * pt + r16, NPIX - 1);
  const int poff = q * PS + (px / OW) * W + (px % OW);
  for (int n = n0; n < n1; n++) {
    const double* img = gt_img + ((n - n0) & 1) * IMG;
    if (n + 1 < n1) stage(gt_img + ((n - n0 + 1) & 1) * IMG);  // (its registers were fetched one image ago)
    if (n + 2 < n1) fetch(n + 2);
    const double* bp = img + poff;
    d4 acc = d4{bz[0], bz[1], bz[2], bz[3]};  // start from the bias: one add less per output
    double bcur = bp[0], bnxt = 0.0;
#pragma unroll
    for (int s = 0; s < NS; s++) {
      if (s + 1 < NS) {
        const int kk = (s + 1) / (C / 4), c4 = (s + 1) % (C / 4);
        bnxt = bp[4 * c4 * PS + (kk / KW) * W + (kk % KW)];
      }
      acc = mfma_f64(a[s], bcur, acc);
      bcur = bnxt;
    }
    if (16 * pt + r16 < NPIX) {
      float* dst = p.O + (((int64_t)n * p.G + g) * F + 16 * ft) * NPIX + 16 * pt + r16;
#pragma unroll
      for (int v = 0; v < 4; v++) store_stream(&dst[(int64_t)d_row(q, v) * NPIX], (float)acc[v]);
    }
    __syncthreads();  // the next image is staged; this image's buffer is free
  }
}

}  // namespace tc355
