// LDS-tiled "NT" contraction for large extents:
//   C[b][n][m] = sum_k A[b][n][k] * Bm[b][m][k]          (+ bias[m], ReLU)
// the path behind tc_tbmm for big matrices -- in particular the paper's transposed
// matmul sizes (Section 7, listing tmm: (M,K,N) up to (128,4096,16384)) -- and
// behind one fcrelu layer (Section 3) when the chain is not run as one kernel.
//
// One workgroup = a 64 x 64 output block, 4 wavefronts of 32 x 32 (2 x 2 MFMA
// tiles).  The reduction is walked in chunks of 32: operand rows are fetched with
// coalesced 16-byte loads two chunks ahead (registers), widened ONCE to fp64 and
// staged in double-buffered LDS ([row][k], row stride 34 doubles, so the 32 lanes
// of an 8-byte read pass hit 64 distinct banks); each k step then needs 2 + 2
// LDS reads for 4 MFMAs and no conversion (a vector-ALU instruction costs
// matrix-pipe time on this chip; widening at staging time is 0.5 conversions per
// MFMA instead of 2).  One barrier per chunk.  Rows past the extents are clamped
// on load and masked on store; the reduction tail is staged as zeros.
// Requires K % 4 == 0 (16-byte loads); other shapes take the wave-level kernel.
#pragma once
#include "gemm_wave.hpp"

namespace tc355 {

constexpr int GT_BM = 64, GT_BN = 64, GT_KC = 32;
constexpr int GT_RS = GT_KC + 2;                               // LDS row stride in doubles: 2*RS = 4 (mod 64) words
constexpr int GT_BUF = (GT_BM + GT_BN) * GT_RS;                // doubles per stage
constexpr int GT_LDS_BYTES = 2 * GT_BUF * 8;                   // 69,632 bytes: two workgroups per compute unit

template <typename TA, int EPI>
__global__ __launch_bounds__(WG_THREADS, 2) void gemm_nt_tile_kernel(GemmArgs p) {
  constexpr bool A64 = sizeof(TA) == 8;
  constexpr int AV = A64 ? 2 : 4;                              // elements of TA per 16-byte load
  constexpr int A_LD = GT_BM * GT_KC / AV / WG_THREADS;         // 16-byte loads per thread and chunk: 2 (fp32) / 4 (fp64)
  constexpr int B_LD = GT_BN * GT_KC / 4 / WG_THREADS;          // 2
  constexpr int A_UPR = GT_KC / AV, B_UPR = GT_KC / 4;          // units per row
  extern __shared__ __attribute__((aligned(16))) double gt_lds[];

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int N = p.N, M = p.M, K = p.K;
  const int tiles_m = (M + GT_BN - 1) / GT_BN;
  const int tn = blockIdx.x / tiles_m, tm = blockIdx.x % tiles_m;  // neighbours share the A rows
  const int64_t b = blockIdx.y;
  const TA* A = static_cast<const TA*>(p.A) + b * p.strideA;
  const float* Bm = p.Bm + b * p.strideB;
  const int n0 = tn * GT_BM, m0 = tm * GT_BN;
  const int nck = (K + GT_KC - 1) / GT_KC;

  // this thread's units of a chunk: rows a_row0 + i*(256/A_UPR), elements a_k..a_k+AV-1 (same for every chunk)
  const int a_row0 = tid / A_UPR, a_k = (tid % A_UPR) * AV;
  const int b_row0 = tid / B_UPR, b_k = (tid % B_UPR) * 4;
  int aoff[A_LD], boff[B_LD];
#pragma unroll
  for (int i = 0; i < A_LD; i++) aoff[i] = min(n0 + a_row0 + i * (WG_THREADS / A_UPR), N - 1) * K + a_k;
#pragma unroll
  for (int i = 0; i < B_LD; i++) boff[i] = min(m0 + b_row0 + i * (WG_THREADS / B_UPR), M - 1) * K + b_k;

  struct Regs {
    Vec<TA, AV> a[A_LD];
    Vec<float, 4> b[B_LD];
  };
  // Loads are never skipped per lane: a unit past K re-reads the start of its row and is staged as zeros.
  auto fetch = [&](Regs& r, int ck) {
    const int k0 = min(ck, nck - 1) * GT_KC;
    if (k0 + GT_KC <= K) {  // whole chunk inside the reduction (uniform): lane offset + scalar base, no ALU work
      const TA* Ak = A + k0;
      const float* Bk = Bm + k0;
#pragma unroll
      for (int i = 0; i < A_LD; i++) r.a[i] = load_vec<TA, AV>(Ak + aoff[i]);
#pragma unroll
      for (int i = 0; i < B_LD; i++) r.b[i] = load_vec<float, 4>(Bk + boff[i]);
    } else {
      const bool ain = k0 + a_k < K, bin = k0 + b_k < K;
#pragma unroll
      for (int i = 0; i < A_LD; i++) r.a[i] = load_vec<TA, AV>(A + aoff[i] + (ain ? k0 : -a_k));
#pragma unroll
      for (int i = 0; i < B_LD; i++) r.b[i] = load_vec<float, 4>(Bm + boff[i] + (bin ? k0 : -b_k));
    }
  };
  auto stage = [&](const Regs& r, int ck, double* buf) {
    const int k0 = ck * GT_KC;
    double* As = buf + a_row0 * GT_RS + a_k;
    double* Bs = buf + GT_BM * GT_RS + b_row0 * GT_RS + b_k;
    if (k0 + GT_KC <= K) {  // whole chunk inside the reduction (uniform): widen and store, nothing else
#pragma unroll
      for (int i = 0; i < A_LD; i++)
#pragma unroll
        for (int e = 0; e < AV; e += 2) {
          dbl2 v = {(double)r.a[i].e[e], (double)r.a[i].e[e + 1]};
          *reinterpret_cast<dbl2*>(As + i * (WG_THREADS / A_UPR) * GT_RS + e) = v;
        }
#pragma unroll
      for (int i = 0; i < B_LD; i++)
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
          dbl2 v = {(double)r.b[i].e[e], (double)r.b[i].e[e + 1]};
          *reinterpret_cast<dbl2*>(Bs + i * (WG_THREADS / B_UPR) * GT_RS + e) = v;
        }
    } else {  // ragged last chunk: what lies past K is staged as zeros
      const bool ain = k0 + a_k < K, bin = k0 + b_k < K;
#pragma unroll
      for (int i = 0; i < A_LD; i++)
#pragma unroll
        for (int e = 0; e < AV; e += 2) {
          dbl2 v = {ain ? (double)r.a[i].e[e] : 0.0, ain ? (double)r.a[i].e[e + 1] : 0.0};
          *reinterpret_cast<dbl2*>(As + i * (WG_THREADS / A_UPR) * GT_RS + e) = v;
        }
#pragma unroll
      for (int i = 0; i < B_LD; i++)
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
          dbl2 v = {bin ? (double)r.b[i].e[e] : 0.0, bin ? (double)r.b[i].e[e + 1] : 0.0};
          *reinterpret_cast<dbl2*>(Bs + i * (WG_THREADS / B_UPR) * GT_RS + e) = v;
        }
    }
  };

  // wavefront (wr, wc) owns rows 32*wr.., columns 32*wc.. of the block
  const int wr = wave >> 1, wc = wave & 1;
  d4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int col = min(m0 + 32 * wc + 16 * j + r16, M - 1);
      // fcrelu's first statement: the output starts as the broadcast bias
      acc[i][j] = (EPI == EPI_BIAS_RELU) ? d4_splat((double)p.bias[col]) : d4_zero();
    }

  // chunk c sits in ring[c % 2] until staged into LDS buffer c % 2; iteration c stages chunk c+1,
  // fetches chunk c+2 and contracts chunk c
  Regs ring[2];
  fetch(ring[0], 0);
  fetch(ring[1], 1);
  stage(ring[0], 0, gt_lds);
  fetch(ring[0], 2);
  __syncthreads();
  for (int c0 = 0; c0 < nck; c0 += 2) {
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int c = c0 + i;
      if (c < nck) {  // uniform
        if (c + 1 < nck) stage(ring[(i + 1) & 1], c + 1, gt_lds + ((i + 1) & 1) * GT_BUF);
        fetch(ring[(i + 1) & 1], c + 3);
        const double* As = gt_lds + (i & 1) * GT_BUF + (32 * wr + r16) * GT_RS + q;
        const double* Bs = gt_lds + (i & 1) * GT_BUF + GT_BM * GT_RS + (32 * wc + r16) * GT_RS + q;
        // LDS reads of step s+1 are issued before the MFMAs of step s (the barriers pin that order;
        // left alone, the compiler reads right before use and the LDS latency lands on the matrix pipe)
        double a0 = As[0], a1 = As[16 * GT_RS], b0 = Bs[0], b1 = Bs[16 * GT_RS];
#pragma unroll
        for (int s = 0; s < GT_KC / 4; s++) {
          double na0 = 0, na1 = 0, nb0 = 0, nb1 = 0;
          if (s + 1 < GT_KC / 4) {
            na0 = As[4 * s + 4]; na1 = As[16 * GT_RS + 4 * s + 4];
            nb0 = Bs[4 * s + 4]; nb1 = Bs[16 * GT_RS + 4 * s + 4];
          }
          __builtin_amdgcn_sched_barrier(0);
          acc[0][0] = mfma_f64(a0, b0, acc[0][0]);
          acc[0][1] = mfma_f64(a0, b1, acc[0][1]);
          acc[1][0] = mfma_f64(a1, b0, acc[1][0]);
          acc[1][1] = mfma_f64(a1, b1, acc[1][1]);
          __builtin_amdgcn_sched_barrier(0);
          a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
        }
        __syncthreads();
      }
    }
  }

  float* C = p.C ? p.C + b * p.strideC : nullptr;
  double* C64 = p.C64 ? p.C64 + b * p.strideC : nullptr;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int col = m0 + 32 * wc + 16 * j + r16;
#pragma unroll
      for (int v = 0; v < 4; v++) {
        const int row = n0 + 32 * wr + 16 * i + d_row(q, v);
        if (row < N && col < M) {
          double x = acc[i][j][v];
          if (EPI == EPI_BIAS_RELU) x = relu64(x);
          const int64_t o = (int64_t)row * M + col;
          if (C) C[o] = (float)x;
          if (C64) C64[o] = x;
        }
      }
    }
}

}  // namespace tc355
