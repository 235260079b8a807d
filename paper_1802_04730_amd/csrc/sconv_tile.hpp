// Strided convolution (Section 3, listing sconv2d):
//   O(n,f,h,w)  = B(f)
//   O(n,f,h,w) += I(n,c, sh*h + kh, sw*w + kw) * W(f,c,kh,kw)
// as an implicit contraction: rows = the F filters, columns = all N*OH*OW
// output pixels of the batch (so that small images still fill whole tiles),
// reduction = the C*KH*KW filter taps in the order W stores them.  The filter
// operand is the row-major [F][C*KH*KW] matrix W itself; the pixel operand is
// gathered from I on the fly: element (tap k, pixel p) lives at
//   pixbase(p) + tapoff(k),  pixbase = (n*C*H + sh*oh)*W + sw*ow,  tapoff = (c*H + kh)*W + kw.
//
// One workgroup = 64 filters x 64 (or 32) pixels, four wavefronts of 32 x 32
// (32 x 16): 2 x 2 (2 x 1) fp64 MFMA tiles; the reduction is walked in chunks of
// 16 taps.  Per chunk a thread gathers 4 (2) input elements (one pixel, taps 4
// (8) apart: consecutive lanes take consecutive pixels, so a wavefront's load
// covers a run of one input row) and one 16-byte piece of a filter row, two
// chunks ahead of the MFMAs; the values are widened once to fp64 and staged in
// double-buffered LDS, filters as [filter][tap] (row stride 18 doubles), pixels
// as [tap][pixel] (row stride 80 (48) doubles: both the 64-lane writes and the
// MFMA operand reads are free of bank conflicts).  Short chunks keep the LDS
// stage under 40 KB, so that three to four workgroups share a compute unit and
// cover each other's gathers (chunks of 32 taps at two workgroups per unit were
// 12-20 % slower).  The (c, kh, kw) of a thread's taps advance by 16 taps per
// chunk with carries instead of divisions.  Accumulators start from the bias, as the
// listing's first statement says.  One barrier per chunk.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

constexpr int SC_BF = 64, SC_KC = 16;
constexpr int SC_RSA = SC_KC + 2;                       // filter stage: row stride in doubles
// BP pixels per block: 64, or 32 when 64 would leave the chip short of blocks
template <int BP>
struct SconvGeom {
  static constexpr int RSB = BP + 16;                          // pixel stage: row stride in doubles, = 16 (mod 32)
  static constexpr int BUF = SC_BF * SC_RSA + SC_KC * RSB;      // doubles per stage
  static constexpr int LDS_BYTES = 2 * BUF * 8;                // 38,912 / 30,720 bytes: four workgroups per compute unit
  static constexpr int TAPS = SC_KC * BP / WG_THREADS;         // gathered elements per thread and chunk: 4 / 2
  static constexpr int KSTEP = WG_THREADS / BP;                // a thread's taps are KSTEP apart: 4 / 8
  static_assert(BP == 64 || BP == 32, "two pixel tiles per wavefront, or one");
};

struct SconvArgs {
  const float* I;     // [N][C][H][W]
  const float* Wt;    // [F][C][KH][KW]
  const float* bias;  // [F] or nullptr
  float* O;           // [N][F][OH][OW]
  int N, C, F, H, W, KH, KW, sh, sw, OH, OW;
  int K;        // C*KH*KW
  int P;        // N*OH*OW
  int tiles_f;  // ceil(F / 64)
};

// AV: floats per load of a filter row (4 needs K % 4 == 0); BP: pixels per block
template <int AV, int BP>
__global__ __launch_bounds__(WG_THREADS, 3) void sconv_tile_kernel(SconvArgs p) {
  using Gm = SconvGeom<BP>;
  constexpr int SC_BP = BP, SC_RSB = Gm::RSB, SC_BUF = Gm::BUF, SC_TAPS = Gm::TAPS, KSTEP = Gm::KSTEP, TJ = BP / 32;
  constexpr int A_LD = SC_BF * SC_KC / AV / WG_THREADS;  // loads per thread and chunk: 2 or 8
  constexpr int A_UPR = SC_KC / AV;                      // units per filter row and chunk
  extern __shared__ __attribute__((aligned(16))) double sc_lds[];
  static_assert(SC_KC % 4 == 0 && SC_KC * BP % WG_THREADS == 0 && SC_BF * SC_KC / AV % WG_THREADS == 0, "whole loads per thread");

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int K = p.K, P = p.P, F = p.F, H = p.H, W = p.W, KH = p.KH, KW = p.KW;
  const int OHW = p.OH * p.OW;
  const int tf = blockIdx.x % p.tiles_f, tp = blockIdx.x / p.tiles_f;  // neighbours share the gathered pixels
  const int f0 = tf * SC_BF, p0 = tp * SC_BP;
  const int nck = (K + SC_KC - 1) / SC_KC;

  // ---- filter rows: units of AV taps, rows a_row0 + i*(256/A_UPR)
  const int a_row0 = tid / A_UPR, a_k = (tid % A_UPR) * AV;
  int aoff[A_LD];
#pragma unroll
  for (int i = 0; i < A_LD; i++) aoff[i] = min(f0 + a_row0 + i * (WG_THREADS / A_UPR), F - 1) * K + a_k;

  // ---- gathered pixels: this thread's pixel, and its taps b_k0 + KSTEP*j of every chunk
  // (with 64 pixels per block a wavefront's lanes share their taps: the tap counters below and the offsets made from
  // them then live in scalar registers and cost the vector ALU nothing)
  const int b_p = tid & (SC_BP - 1), b_k0 = SC_BP == WAVE ? wave : tid / SC_BP;
  int pixbase;
  {
    const int px = min(p0 + b_p, P - 1);  // clamped: a ragged tile re-reads the last pixel and does not store it
    const int n = px / OHW, r = px - n * OHW;
    const int oh = r / p.OW, ow = r - oh * p.OW;
    pixbase = (n * p.C * H + p.sh * oh) * W + p.sw * ow;
  }
  // taps as (c, kh, kw) with carries; one chunk further = + (dc, dkh, dkw)
  int tc[SC_TAPS], tkh[SC_TAPS], tkw[SC_TAPS];
#pragma unroll
  for (int j = 0; j < SC_TAPS; j++) {
    const int k = b_k0 + KSTEP * j;
    tkw[j] = k % KW;
    tkh[j] = (k / KW) % KH;
    tc[j] = k / (KW * KH);
  }
  const int dkw = SC_KC % KW, dkh = (SC_KC / KW) % KH, dc = SC_KC / (KW * KH);

  struct Regs {
    Vec<float, AV> a[A_LD];
    float b[SC_TAPS];
  };
  // fetch the chunk the tap counters stand at, then advance them
  int fck = 0;
  auto fetch = [&](Regs& r) {
    const int k0 = min(fck, nck - 1) * SC_KC;
    const bool whole = k0 + SC_KC <= K;  // uniform
    if (whole) {  // every chunk but perhaps the last: no per-lane choice at all
#pragma unroll
      for (int i = 0; i < A_LD; i++) r.a[i] = load_vec<float, AV>(p.Wt + aoff[i] + k0);
#pragma unroll
      for (int j = 0; j < SC_TAPS; j++) r.b[j] = p.I[pixbase + ((tc[j] * H + tkh[j]) * W + tkw[j])];
    } else {
#pragma unroll
      for (int i = 0; i < A_LD; i++) r.a[i] = load_vec<float, AV>(p.Wt + aoff[i] + (k0 + a_k < K ? k0 : -a_k));
#pragma unroll
      for (int j = 0; j < SC_TAPS; j++) {
        const bool in = k0 + b_k0 + KSTEP * j < K;
        r.b[j] = p.I[pixbase + (in ? (tc[j] * H + tkh[j]) * W + tkw[j] : 0)];  // a tap past K reads a valid element, staged as 0
      }
    }
    if (fck + 1 < nck) {
#pragma unroll
      for (int j = 0; j < SC_TAPS; j++) {
        tkw[j] += dkw;
        if (tkw[j] >= KW) { tkw[j] -= KW; tkh[j]++; }
        tkh[j] += dkh;
        if (tkh[j] >= KH) { tkh[j] -= KH; tc[j]++; }
        tc[j] += dc;
      }
    }
    fck++;
  };
  auto stage = [&](const Regs& r, int ck, double* buf) {
    const int k0 = ck * SC_KC;
    const bool whole = k0 + SC_KC <= K;
    double* As = buf + a_row0 * SC_RSA + a_k;
    double* Bs = buf + SC_BF * SC_RSA + b_k0 * SC_RSB + b_p;
    if (whole) {  // (uniform)
#pragma unroll
      for (int i = 0; i < A_LD; i++) {
        if constexpr (AV == 4) {
#pragma unroll
          for (int e = 0; e < 4; e += 2) {
            dbl2 v = {(double)r.a[i].e[e], (double)r.a[i].e[e + 1]};
            *reinterpret_cast<dbl2*>(As + i * (WG_THREADS / A_UPR) * SC_RSA + e) = v;
          }
        } else {
          As[i * (WG_THREADS / A_UPR) * SC_RSA] = (double)r.a[i].e[0];
        }
      }
#pragma unroll
      for (int j = 0; j < SC_TAPS; j++) Bs[KSTEP * j * SC_RSB] = (double)r.b[j];
      return;
    }
    const bool ain = k0 + a_k < K;
#pragma unroll
    for (int i = 0; i < A_LD; i++) {
      if constexpr (AV == 4) {
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
          dbl2 v = {ain ? (double)r.a[i].e[e] : 0.0, ain ? (double)r.a[i].e[e + 1] : 0.0};
          *reinterpret_cast<dbl2*>(As + i * (WG_THREADS / A_UPR) * SC_RSA + e) = v;
        }
      } else {
        As[i * (WG_THREADS / A_UPR) * SC_RSA] = ain ? (double)r.a[i].e[0] : 0.0;
      }
    }
#pragma unroll
    for (int j = 0; j < SC_TAPS; j++) {
      const bool in = k0 + b_k0 + KSTEP * j < K;
      Bs[KSTEP * j * SC_RSB] = in ? (double)r.b[j] : 0.0;
    }
  };

  // wavefront (wr, wc) owns filters 32*wr.., pixels 16*TJ*wc.. of the block
  const int wr = wave >> 1, wc = wave & 1;
  d4 acc[2][TJ];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    d4 bz;
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const int f = min(f0 + 32 * wr + 16 * i + d_row(q, v), F - 1);
      bz[v] = p.bias ? (double)p.bias[f] : 0.0;  // the listing's first statement
    }
#pragma unroll
    for (int j = 0; j < TJ; j++) acc[i][j] = bz;
  }

  // chunk c sits in ring[c % 2] until staged into LDS buffer c % 2; iteration c stages chunk c+1,
  // fetches chunk c+2 and contracts chunk c
  Regs ring[2];
  fetch(ring[0]);
  fetch(ring[1]);
  stage(ring[0], 0, sc_lds);
  fetch(ring[0]);
  __syncthreads();
  for (int c0 = 0; c0 < nck; c0 += 2) {
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int c = c0 + i;
      if (c < nck) {  // uniform
        if (c + 1 < nck) stage(ring[(i + 1) & 1], c + 1, sc_lds + ((i + 1) & 1) * SC_BUF);
        fetch(ring[(i + 1) & 1]);
        const double* As = sc_lds + (i & 1) * SC_BUF + (32 * wr + r16) * SC_RSA + q;
        const double* Bs = sc_lds + (i & 1) * SC_BUF + SC_BF * SC_RSA + q * SC_RSB + 16 * TJ * wc + r16;
        // LDS reads of step s+1 are issued before the MFMAs of step s
        double a0 = As[0], a1 = As[16 * SC_RSA], b[TJ], nb[TJ];
#pragma unroll
        for (int j = 0; j < TJ; j++) b[j] = Bs[16 * j];
#pragma unroll
        for (int s = 0; s < SC_KC / 4; s++) {
          double na0 = 0, na1 = 0;
          if (s + 1 < SC_KC / 4) {
            na0 = As[4 * s + 4]; na1 = As[16 * SC_RSA + 4 * s + 4];
#pragma unroll
            for (int j = 0; j < TJ; j++) nb[j] = Bs[(4 * s + 4) * SC_RSB + 16 * j];
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int j = 0; j < TJ; j++) acc[0][j] = mfma_f64(a0, b[j], acc[0][j]);
#pragma unroll
          for (int j = 0; j < TJ; j++) acc[1][j] = mfma_f64(a1, b[j], acc[1][j]);
          __builtin_amdgcn_sched_barrier(0);
          a0 = na0; a1 = na1;
#pragma unroll
          for (int j = 0; j < TJ; j++) b[j] = nb[j];
        }
        __syncthreads();
      }
    }
  }

#pragma unroll
  for (int j = 0; j < TJ; j++) {
    const int px = p0 + 16 * TJ * wc + 16 * j + r16;
    const int pc = min(px, P - 1);
    const int n = pc / OHW, r = pc - n * OHW;
    float* out = p.O + (int64_t)n * F * OHW + r;
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int v = 0; v < 4; v++) {
        const int f = f0 + 32 * wr + 16 * i + d_row(q, v);
        if (px < P && f < F) out[(int64_t)f * OHW] = (float)acc[i][j][v];
      }
  }
}

}  // namespace tc355
