// Tuned Kronecker-factored layer (benchmark configuration 5) for compile-time
// K, L, J that are multiples of 16:
//   T(b,i,l) = sum_k W1(i,k) X(b,k,l)     then     Y(b,i,j) = sum_l T(b,i,l) W2(j,l).
//
// One workgroup (4 wavefronts) owns one batch element and 64 rows i; wavefront
// w owns rows 16w..16w+15.  X_b and W2 are staged once into LDS, WIDENED to fp64
// on the way in (a vector-ALU instruction costs matrix-pipe time on this chip, and
// widening at staging time takes 32 conversions per thread instead of 256 inside
// the MFMA loop), with row strides of L+4 and L+2 doubles, which spread the 32
// lanes of every 8-byte operand read pass over 64 distinct banks.  The W1 rows
// of a wavefront live in registers as fp64.
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
  constexpr int LS = L + 4;   // LDS row stride (doubles) of X_b:  8*LS  = 32 (mod 64) words between k slots
  constexpr int LS2 = L + 2;  // LDS row stride (doubles) of W2:   2*LS2 =  4 (mod 64) words between rows
  constexpr int TJ = J / 16;  // output column tiles
  __shared__ __attribute__((aligned(16))) double Xs[K * LS];
  __shared__ __attribute__((aligned(16))) double W2s[J * LS2];

  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1), wave = tid / WAVE;
  const int r16 = lane & 15, q = lane >> 4;
  const int ib = blockIdx.x % p.iblocks;
  const int64_t b = blockIdx.x / p.iblocks;
  const int I = p.I;
  const int i0 = ib * 64 + wave * 16;

  // ---- stage X_b and W2 (coalesced 16-byte loads)
  const float* X = p.X + b * (int64_t)K * L;
  constexpr int XU = K * L / 2 / WG_THREADS, WU = J * L / 2 / WG_THREADS;  // 8-byte units per thread
  static_assert((K * L / 2) % WG_THREADS == 0 && (J * L / 2) % WG_THREADS == 0, "whole units per thread");
  f2 xpre[XU], wpre[WU];  // all loads first, then the LDS writes (consecutive lanes write consecutive 16 bytes)
#pragma unroll
  for (int u = 0; u < XU; u++) xpre[u] = *reinterpret_cast<const f2*>(X + 2 * (tid + u * WG_THREADS));
#pragma unroll
  for (int u = 0; u < WU; u++) wpre[u] = *reinterpret_cast<const f2*>(p.W2 + 2 * (tid + u * WG_THREADS));
  // ---- W1 rows of this wavefront: lane holds W1[i0+r16][16j + 4q + e]
  f4 w1f[K / 16];
  {
    const float* w1p = p.W1 + (int64_t)min(i0 + r16, I - 1) * K + 4 * q;
#pragma unroll
    for (int j = 0; j < K / 16; j++) w1f[j] = *reinterpret_cast<const f4*>(w1p + 16 * j);
  }
#pragma unroll
  for (int u = 0; u < XU; u++) {
    const int idx = tid + u * WG_THREADS, r = idx / (L / 2), c = idx - r * (L / 2);
    dbl2 v = {(double)xpre[u][0], (double)xpre[u][1]};
    *reinterpret_cast<dbl2*>(Xs + r * LS + 2 * c) = v;
  }
#pragma unroll
  for (int u = 0; u < WU; u++) {
    const int idx = tid + u * WG_THREADS, r = idx / (L / 2), c = idx - r * (L / 2);
    dbl2 v = {(double)wpre[u][0], (double)wpre[u][1]};
    *reinterpret_cast<dbl2*>(W2s + r * LS2 + 2 * c) = v;
  }
  double w1[K / 16][4];
#pragma unroll
  for (int j = 0; j < K / 16; j++)
#pragma unroll
    for (int e = 0; e < 4; e++) w1[j][e] = (double)w1f[j][e];
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
        Tt = mfma_f64(Xs[(16 * j + 4 * q + e) * LS + l0 + r16], w1[j][e], Tt);
      }
    // second contraction: step v consumes l = l0 + 4v + q
#pragma unroll
    for (int v = 0; v < 4; v++)
#pragma unroll
      for (int t = 0; t < TJ; t++) {
        acc[t] = mfma_f64(Tt[v], W2s[(16 * t + r16) * LS2 + l0 + 4 * v + q], acc[t]);
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
