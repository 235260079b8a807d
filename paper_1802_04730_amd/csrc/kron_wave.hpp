// Shape-generic Kronecker-factored layer (benchmark configuration 5):
//   Y(b,i,j) = sum_{k,l} W1(i,k) * W2(j,l) * X(b,k,l)
// evaluated as two chained contractions,
//   T(b,i,l) = sum_k W1(i,k) X(b,k,l)      then      Y(b,i,j) = sum_l T(b,i,l) W2(j,l),
// with T kept in the MFMA accumulator registers in fp64.
//
// One wavefront owns 16 rows i of one batch element and up to 16*TJ columns j.
// For each block of 16 values of l it computes the TRANSPOSED tile
// T^t[l][i] = sum_k X[k][l] * W1[i][k]; in the MFMA result layout a lane then
// holds T[i = r16][l = l0 + 4v + q], which is exactly what the A operand of
// the second contraction needs (row r16, k slot q) if step v of that
// contraction consumes l = l0 + 4v + q.  So the intermediate never moves.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct KronArgs {
  const float* W1;  // [I][K]
  const float* W2;  // [J][L]
  const float* X;   // [B][K][L]
  float* Y;         // [B][I][J]
  int I, K, J, L;
  int tiles_i;   // ceil(I / 16)
  int blocks_j;  // ceil(J / (16*TJ))
  int64_t jobs;  // B * tiles_i * blocks_j
};

template <int TJ>
__global__ __launch_bounds__(WG_THREADS) void kron_wave_kernel(KronArgs p) {
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const int r16 = lane & 15, q = lane >> 4;
  const int64_t job = (int64_t)blockIdx.x * WAVES_PER_WG + wave;
  if (job >= p.jobs) return;

  const int bj = (int)(job % p.blocks_j);
  const int64_t rest = job / p.blocks_j;
  const int ti = (int)(rest % p.tiles_i);
  const int64_t b = rest / p.tiles_i;
  const int I = p.I, K = p.K, J = p.J, L = p.L;
  const int i0 = ti * 16, j0 = bj * 16 * TJ;

  const float* X = p.X + b * (int64_t)K * L;
  const float* w1p = p.W1 + (int64_t)min(i0 + r16, I - 1) * K;
  const float* w2p[TJ];
#pragma unroll
  for (int t = 0; t < TJ; t++) w2p[t] = p.W2 + (int64_t)min(j0 + 16 * t + r16, J - 1) * L;

  d4 acc[TJ];
#pragma unroll
  for (int t = 0; t < TJ; t++) acc[t] = d4_zero();

  for (int l0 = 0; l0 < L; l0 += 16) {
    // stage 1: Tt[v] = T[i0 + r16][l0 + 4v + q]
    d4 Tt = d4_zero();
    const int la = l0 + r16;
    const bool lin = la < L;
    for (int k0 = 0; k0 < K; k0 += 4) {
      const int kk = k0 + q;
      const bool kin = kk < K;
      const double a = (kin && lin) ? (double)X[(int64_t)kk * L + la] : 0.0;
      const double bb = kin ? (double)w1p[kk] : 0.0;
      Tt = mfma_f64(a, bb, Tt);
    }
    // stage 2: step v consumes l = l0 + 4v + q
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const int l = l0 + 4 * v + q;
      const bool in = l < L;
      const double a2 = in ? Tt[v] : 0.0;
#pragma unroll
      for (int t = 0; t < TJ; t++) {
        const double b2 = in ? (double)w2p[t][in ? l : 0] : 0.0;
        acc[t] = mfma_f64(a2, b2, acc[t]);
      }
    }
  }

  float* Y = p.Y + b * (int64_t)I * J;
#pragma unroll
  for (int t = 0; t < TJ; t++) {
    const int j = j0 + 16 * t + r16;
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const int i = i0 + d_row(q, v);
      if (i < I && j < J) Y[(int64_t)i * J + j] = (float)acc[t][v];
    }
  }
}

}  // namespace tc355
