// Transposed batched matmul for SMALL per-batch matrices (Section 7, "Transposed
// Batched Matrix Multiplication", listing tbmm; the benchmark's 26 x 72 x 26):
//
//     Z(b,n,m) = sum_k X(b,n,k) * Y(b,m,k)
//
// A job is one batch element b, a strip of 16*TN rows of X_b and a strip of
// 16*TM rows of Y_b.  Both strips are contiguous in memory (the reduction index
// is the fastest one and a strip takes whole rows), so a wavefront copies them
// as flat streams of 16-byte pieces (every load instruction of the wavefront
// fetches 1 KiB of consecutive addresses), parks them unchanged in its private
// LDS region and feeds the fp64 matrix core from there: lane (r16, q) of step s
// reads element k = 4s + q of its row as one 4-byte LDS read and widens it.
// Nothing is shared between wavefronts, so there is no barrier; a wavefront
// walks over its jobs and has the global loads of its next DEPTH jobs in flight
// (in registers) while it contracts the current one.
//
// MFMA roles: A = Y rows (result rows = m), B = X rows (result columns = n).
// Result row i of a tile is made to carry m = 4*(i%4) + i/4 of the tile (just a
// choice of which Y row a lane reads), so the four accumulator values of a lane
// are four CONSECUTIVE m of one n: 16 bytes of a row of Z.
//
// Write-back.  When the Y strip covers all of M (and M is a multiple of 4), the
// job's part of Z is one contiguous block: the 16-byte pieces go through the
// (now idle) LDS region and leave as flat 1 KiB streaming stores per
// instruction.  (Measured on the memory skeleton of this kernel at B = 32000:
// flat streaming stores 93 us, flat plain stores 106 us, 64-byte pieces of 16
// rows per instruction 113 us plain and 133-150 us streaming.)  Otherwise a lane
// stores its pieces directly with plain stores.
//
// Requirements (checked by the host): N*K and M*K multiples of 4 (every strip
// then starts and ends on a 16-byte boundary); a strip of X takes at most NX
// load instructions (64 pieces each) and a strip of Y at most NY; the regions
// of a workgroup fit the LDS.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct TbmmLdsArgs {
  const float* X;  // [B][N][K]
  const float* Y;  // [B][M][K]
  float* Z;        // [B][N][M]
  int N, M, K;
  int strips_n;        // ceil(N / (16*TN))
  int strips_m;        // ceil(M / (16*TM))
  int jobs;            // B * strips_n * strips_m  (< 2^31, checked by the host)
  int wave_lds_units;  // 16-byte units of LDS per wavefront
};

// How a job's results leave: as one contiguous block through LDS (the Y strip covers all of M, M a multiple of 4),
// as 16-byte pieces straight from the accumulators (M a multiple of 4), or element by element.
enum { TBMM_STORE_FLAT = 0, TBMM_STORE_PIECES = 1, TBMM_STORE_SCALAR = 2 };

// KS: number of 4-element reduction steps if known at compile time (K in 4*KS-3 .. 4*KS), else 0.
template <int TN, int TM, int NX, int NY, int DEPTH, int STORE, int KS>
__global__ __launch_bounds__(WG_THREADS, 2) void tbmm_lds_kernel(TbmmLdsArgs p) {
  extern __shared__ __attribute__((aligned(16))) char tbmm_smem[];
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int N = p.N, M = p.M, K = p.K;
  char* lds = tbmm_smem + (size_t)wave * p.wave_lds_units * 16;
  const float* ldsf = reinterpret_cast<const float*>(lds);
  const unsigned stride = gridDim.x * WAVES_PER_WG;
  unsigned job = blockIdx.x * WAVES_PER_WG + wave;
  if (job >= (unsigned)p.jobs) return;  // whole wavefront leaves together; there is no barrier in this kernel

  struct Geo {
    unsigned b;
    int n0, m0;
    int xu, yu;  // 16-byte pieces of the X strip and of the Y strip
  };
  auto geometry = [&](unsigned j) {
    Geo g;
    const unsigned rest = j / (unsigned)p.strips_m;
    const int sm = (int)(j - rest * (unsigned)p.strips_m);
    g.b = rest / (unsigned)p.strips_n;
    const int sn = (int)(rest - g.b * (unsigned)p.strips_n);
    g.n0 = sn * 16 * TN;
    g.m0 = sm * 16 * TM;
    g.xu = (min(16 * TN, N - g.n0) * K) >> 2;
    g.yu = (min(16 * TM, M - g.m0) * K) >> 2;
    return g;
  };
  // Load instruction i < NX fetches pieces 64*i .. 64*i+63 of the X strip, instruction NX + i those of the Y strip;
  // lanes past the end of a strip repeat its last piece (same address, same value, same LDS slot), so no load and no
  // LDS write sits in a per-lane branch.  An address is a uniform base plus a 32-bit byte offset per lane.
  struct Pre {
    f4 x[NX];
    f4 y[NY];
  };
  auto fetch = [&](const Geo& g, Pre& r) {
    const char* xs = reinterpret_cast<const char*>(p.X + ((int64_t)g.b * N + g.n0) * K);
    const char* ys = reinterpret_cast<const char*>(p.Y + ((int64_t)g.b * M + g.m0) * K);
#pragma unroll
    for (int i = 0; i < NX; i++) r.x[i] = *reinterpret_cast<const f4*>(xs + 16u * (unsigned)min(i * WAVE + lane, g.xu - 1));
#pragma unroll
    for (int i = 0; i < NY; i++) r.y[i] = *reinterpret_cast<const f4*>(ys + 16u * (unsigned)min(i * WAVE + lane, g.yu - 1));
  };
  auto park = [&](const Geo& g, const Pre& r) {
#pragma unroll
    for (int i = 0; i < NX; i++) *reinterpret_cast<f4*>(lds + 16 * min(i * WAVE + lane, g.xu - 1)) = r.x[i];
#pragma unroll
    for (int i = 0; i < NY; i++) *reinterpret_cast<f4*>(lds + 16 * (g.xu + min(i * WAVE + lane, g.yu - 1))) = r.y[i];
  };

  const int ksteps = (K + 3) >> 2;

  // ring of prefetched jobs: slot d holds job + d*stride
  Geo geo[DEPTH];
  Pre pre[DEPTH];
#pragma unroll
  for (int d = 0; d < DEPTH; d++) {
    const unsigned j = job + d * stride;
    if (j < (unsigned)p.jobs && j >= job) {
      geo[d] = geometry(j);
      fetch(geo[d], pre[d]);
    }
  }
  for (;;) {
#pragma unroll
    for (int d = 0; d < DEPTH; d++) {
      if (job >= (unsigned)p.jobs) return;  // uniform
      const Geo g = geo[d];
      park(g, pre[d]);
      {
        const unsigned ahead = job + DEPTH * stride;
        if (ahead < (unsigned)p.jobs && ahead > job) {  // uniform
          geo[d] = geometry(ahead);
          fetch(geo[d], pre[d]);  // in flight while this and the next DEPTH-1 jobs are contracted
        }
      }

      // LDS float index of element k = q of this lane's rows (row clamped into the strip; such rows are never stored)
      int aidx[TM], bidx[TN];
#pragma unroll
      for (int t = 0; t < TM; t++) {
        const int ml = 16 * t + 4 * (r16 & 3) + (r16 >> 2);
        aidx[t] = 4 * g.xu + min(ml, M - 1 - g.m0) * K + q;
      }
#pragma unroll
      for (int t = 0; t < TN; t++) bidx[t] = min(16 * t + r16, N - 1 - g.n0) * K + q;

      d4 acc[TN][TM];
#pragma unroll
      for (int tn = 0; tn < TN; tn++)
#pragma unroll
        for (int tm = 0; tm < TM; tm++) acc[tn][tm] = d4_zero();

      // One step = 4 reduction elements: TM + TN LDS reads, as many conversions, TM*TN MFMAs.  In the last step of
      // a reduction that is not a multiple of 4 the slots past K are zeroed in BOTH operands: what was read there
      // is the next row's data, possibly an Inf.
      auto step = [&](int s, bool last) {
        float af[TM], bf[TN];
#pragma unroll
        for (int t = 0; t < TM; t++) af[t] = ldsf[aidx[t] + 4 * s];
#pragma unroll
        for (int t = 0; t < TN; t++) bf[t] = ldsf[bidx[t] + 4 * s];
        if (last && 4 * s + q >= K) {
#pragma unroll
          for (int t = 0; t < TM; t++) af[t] = 0.0f;
#pragma unroll
          for (int t = 0; t < TN; t++) bf[t] = 0.0f;
        }
#pragma unroll
        for (int tm = 0; tm < TM; tm++)
#pragma unroll
          for (int tn = 0; tn < TN; tn++) acc[tn][tm] = mfma_f64((double)af[tm], (double)bf[tn], acc[tn][tm]);
      };
      if constexpr (KS > 0) {  // compile-time step count: LDS reads at immediate offsets, scheduled freely
#pragma unroll
        for (int s = 0; s < KS; s++) step(s, s == KS - 1);
      } else {
        for (int s = 0; s < ksteps - 1; s++) step(s, false);
        step(ksteps - 1, true);
      }

      // write-back: Z[b][n0 + 16*tn + r16][m0 + 16*tm + 4*q + v] = acc[tn][tm][v]
      if constexpr (STORE == TBMM_STORE_FLAT) {
        // rows n0 .. n0+rows-1 of Z_b, all M columns: one contiguous block, laid out in the LDS region first
        const int rows = min(16 * TN, N - g.n0);
#pragma unroll
        for (int tn = 0; tn < TN; tn++)
#pragma unroll
          for (int tm = 0; tm < TM; tm++) {
            const d4 x = acc[tn][tm];
            const f4 o = {(float)x[0], (float)x[1], (float)x[2], (float)x[3]};
            if (16 * tn + r16 < rows && 16 * tm + 4 * q < M)
              *reinterpret_cast<f4*>(lds + 4 * ((16 * tn + r16) * M + 16 * tm + 4 * q)) = o;
          }
        const int zu = (rows * M) >> 2;
        f4* zs = reinterpret_cast<f4*>(p.Z + ((int64_t)g.b * N + g.n0) * M);
#pragma unroll
        for (int i = 0; i < TN * TM; i++) {
          const int u = i * WAVE + lane;
          if (u < zu) store_stream(zs + u, *reinterpret_cast<const f4*>(lds + 16 * u));
        }
      } else {
        float* Zl = p.Z + ((int64_t)g.b * N + g.n0 + r16) * M + g.m0 + 4 * q;  // this lane's piece of tile (0, 0)
        if constexpr (STORE == TBMM_STORE_PIECES) {  // a piece is wholly inside or wholly outside
#pragma unroll
          for (int tn = 0; tn < TN; tn++)
#pragma unroll
            for (int tm = 0; tm < TM; tm++) {
              const d4 x = acc[tn][tm];
              const f4 o = {(float)x[0], (float)x[1], (float)x[2], (float)x[3]};
              if (g.n0 + 16 * tn + r16 < N && g.m0 + 16 * tm + 4 * q < M)
                *reinterpret_cast<f4*>(Zl + (int64_t)tn * 16 * M + 16 * tm) = o;
            }
        } else {
#pragma unroll
          for (int tn = 0; tn < TN; tn++)
#pragma unroll
            for (int tm = 0; tm < TM; tm++)
#pragma unroll
              for (int v = 0; v < 4; v++)
                if (g.n0 + 16 * tn + r16 < N && g.m0 + 16 * tm + 4 * q + v < M)
                  Zl[(int64_t)tn * 16 * M + 16 * tm + v] = (float)acc[tn][tm][v];
        }
      }
      const unsigned next = job + stride;
      if (next <= job) return;  // 32-bit wrap: no further job
      job = next;
    }
  }
}

}  // namespace tc355
