// Tuned Kronecker-factored layer (benchmark configuration 5) for compile-time
// K, L, J that are multiples of 16:
//   T(b,i,l) = sum_k W1(i,k) X(b,k,l)     then     Y(b,i,j) = sum_l T(b,i,l) W2(j,l).
//
// One workgroup (4 wavefronts) owns one batch element and 64 rows i; wavefront
// w owns rows 16w..16w+15.  X_b and W2 are staged once into LDS as fp32 with a
// row stride of L+4 words, which spreads the 64 lanes of every MFMA operand
// read over 64 distinct banks.  The W1 rows of a wavefront live in registers.
// The first contraction is computed transposed, so its result tile already
// sits in the lanes/registers where the second contraction wants its A
// operand: T never leaves the register file and is never rounded.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct KronLdsArgs {
  const float* W1;  // [I][K]
  const float* W2;  // [J][L]
  const float* X;   // [B][K][L]
  float* Y;         // [B][I][J]
  int I;
  int iblocks;  // ceil(I / 64)
};

template <int K, int L, int J>
__global__ __launch_bounds__(WG_THREADS) void kron_lds_kernel(KronLdsArgs p) {
  static_assert(K % 16 == 0 && L % 16 == 0 && J % 16 == 0, "extents must be multiples of 16");
  constexpr int LS = L + 4;   // LDS row stride (floats) of X_b and of W2
  constexpr int TJ = J / 16;  // output column tiles
  __shared__ __attribute__((aligned(16))) float Xs[K * LS];
  __shared__ __attribute__((aligned(16))) float W2s[J * LS];

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1), wave = tid / WAVE;
  const int r16 = lane & 15, q = lane >> 4;
  const int ib = blockIdx.x % p.iblocks;
  const int64_t b = blockIdx.x / p.iblocks;
  const int I = p.I;
  const int i0 = ib * 64 + wave * 16;

  // ---- stage X_b and W2 (coalesced 16-byte loads)
  const float* X = p.X + b * (int64_t)K * L;
  for (int idx = tid; idx < K * L / 4; idx += WG_THREADS) {
    const int r = idx / (L / 4), c = idx - r * (L / 4);
    *reinterpret_cast<f4*>(Xs + r * LS + 4 * c) = *reinterpret_cast<const f4*>(X + r * L + 4 * c);
  }
  for (int idx = tid; idx < J * L / 4; idx += WG_THREADS) {
    const int r = idx / (L / 4), c = idx - r * (L / 4);
    *reinterpret_cast<f4*>(W2s + r * LS + 4 * c) = *reinterpret_cast<const f4*>(p.W2 + r * L + 4 * c);
  }
  // ---- W1 rows of this wavefront: lane holds W1[i0+r16][16j + 4q + e]
  f4 w1[K / 16];
  {
    const float* w1p = p.W1 + (int64_t)min(i0 + r16, I - 1) * K + 4 * q;
#pragma unroll
    for (int j = 0; j < K / 16; j++) w1[j] = *reinterpret_cast<const f4*>(w1p + 16 * j);
  }
  __syncthreads();
  if (i0 >= I) return;  // no barrier follows

  d4 acc[TJ];
#pragma unroll
  for (int t = 0; t < TJ; t++) acc[t] = d4_zero();

#pragma unroll
  for (int lt = 0; lt < L / 16; lt++) {
    const int l0 = 16 * lt;
    // first contraction, transposed: Tt[v] = T[i0 + r16][l0 + 4v + q]
    d4 Tt = d4_zero();
#pragma unroll
    for (int j = 0; j < K / 16; j++)
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const double a = (double)Xs[(16 * j + 4 * q + e) * LS + l0 + r16];
        Tt = mfma_f64(a, (double)w1[j][e], Tt);
      }
    // second contraction: step v consumes l = l0 + 4v + q
#pragma unroll
    for (int v = 0; v < 4; v++)
#pragma unroll
      for (int t = 0; t < TJ; t++) {
        const double b2 = (double)W2s[(16 * t + r16) * LS + l0 + 4 * v + q];
        acc[t] = mfma_f64(Tt[v], b2, acc[t]);
      }
  }

  float* Y = p.Y + b * (int64_t)I * J;
#pragma unroll
  for (int v = 0; v < 4; v++) {
    const int i = i0 + d_row(q, v);
    if (i < I) {
#pragma unroll
      for (int t = 0; t < TJ; t++) Y[(int64_t)i * J + 16 * t + r16] = (float)acc[t][v];
    }
  }
}

}  // namespace tc355
