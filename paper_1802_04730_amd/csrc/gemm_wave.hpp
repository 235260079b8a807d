// Wave-level "NT" contraction  C[b][n][m] = sum_k A[b][n][k] * Bm[b][m][k]
// for arbitrary extents: the shape-generic path behind tc_tbmm (Section 7,
// listing tbmm) and behind one fcrelu layer (Section 3, listing fcrelu).
//
// One wavefront owns a 16 x (16*TM) strip of one batch element's output and
// feeds the fp64 MFMA straight from global memory: no LDS, no barrier, so the
// only dependency chain is load -> widen -> MFMA -> store.  Rows/columns past
// the extents are clamped on load and masked on store; reduction slots past K
// are zeroed in BOTH operands (a clamped load may fetch an Inf, and 0*Inf
// would poison the sum).
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

struct GemmArgs {
  const void* A;      // [batch][N][K], float or double (template TA)
  const float* Bm;    // [batch][M][K]
  const float* bias;  // [M] (EPI_BIAS_RELU) or unused
  float* C;           // [batch][N][M] fp32 result, or nullptr
  double* C64;        // [batch][N][M] fp64 copy for a following stage, or nullptr
  int64_t strideA, strideB, strideC;  // elements between batch entries
  int N, M, K;
  int tiles_n;   // ceil(N / 16)
  int strips_m;  // ceil(M / (16*TM))
  int64_t jobs;  // batch * tiles_n * strips_m
};

enum { EPI_NONE = 0, EPI_BIAS_RELU = 1 };

// VEC consecutive reduction elements are fetched per lane and load; k slot q
// of MFMA step e then carries element k0 + VEC*q + e.  Requires K % VEC == 0.
template <typename TA, int VEC, int TM, int EPI>
__global__ __launch_bounds__(WG_THREADS) void gemm_nt_wave_kernel(GemmArgs p) {
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const int r16 = lane & 15, q = lane >> 4;
  const int64_t job = (int64_t)blockIdx.x * WAVES_PER_WG + wave;
  if (job >= p.jobs) return;  // whole wavefront leaves together; no barrier follows

  const int sm = (int)(job % p.strips_m);
  const int64_t rest = job / p.strips_m;
  const int tn = (int)(rest % p.tiles_n);
  const int64_t b = rest / p.tiles_n;
  const int N = p.N, M = p.M, K = p.K;
  const int n0 = tn * 16, m0 = sm * 16 * TM;

  const TA* A = static_cast<const TA*>(p.A) + b * p.strideA;
  const float* Bm = p.Bm + b * p.strideB;
  const int arow = min(n0 + r16, N - 1);
  const TA* ap = A + (int64_t)arow * K;
  const float* bp[TM];
  d4 acc[TM];
#pragma unroll
  for (int t = 0; t < TM; t++) {
    const int bcol = min(m0 + 16 * t + r16, M - 1);
    bp[t] = Bm + (int64_t)bcol * K;
    // fcrelu's first statement: the output starts as the broadcast bias
    acc[t] = (EPI == EPI_BIAS_RELU) ? d4_splat((double)p.bias[bcol]) : d4_zero();
  }

  // The reduction is walked in chunks of 4*VEC elements; GC chunks form a group and
  // the loads of group g+1 are issued before the MFMAs of group g, so several
  // memory round trips are in flight per wavefront at any time.
  constexpr int GC = 4;
  constexpr int CH = 4 * VEC;
  struct Chunk {
    Vec<TA, VEC> a;
    Vec<float, VEC> b[TM];
  };
  auto load_chunk = [&](int k0, Chunk& c) {
    const int kk = k0 + VEC * q;
    const int kc = kk < K ? kk : 0;
    c.a = load_vec<TA, VEC>(ap + kc);
#pragma unroll
    for (int t = 0; t < TM; t++) c.b[t] = load_vec<float, VEC>(bp[t] + kc);
  };
  auto compute_chunk = [&](int k0, const Chunk& c) {
    if (k0 >= K) return;  // uniform over the wavefront
    const bool in = k0 + VEC * q < K;
#pragma unroll
    for (int e = 0; e < VEC; e++) {
      const double a = in ? (double)c.a.e[e] : 0.0;
#pragma unroll
      for (int t = 0; t < TM; t++) {
        const double bb = in ? (double)c.b[t].e[e] : 0.0;
        acc[t] = mfma_f64(a, bb, acc[t]);
      }
    }
  };
  Chunk cur[GC], nxt[GC];
#pragma unroll
  for (int i = 0; i < GC; i++) load_chunk(i * CH, cur[i]);
  for (int k0 = 0; k0 < K; k0 += GC * CH) {
    const bool more = k0 + GC * CH < K;
    if (more) {
#pragma unroll
      for (int i = 0; i < GC; i++) load_chunk(k0 + (GC + i) * CH, nxt[i]);
    }
#pragma unroll
    for (int i = 0; i < GC; i++) compute_chunk(k0 + i * CH, cur[i]);
    if (more) {
#pragma unroll
      for (int i = 0; i < GC; i++) cur[i] = nxt[i];
    }
  }

  float* C = p.C ? p.C + b * p.strideC : nullptr;
  double* C64 = p.C64 ? p.C64 + b * p.strideC : nullptr;
#pragma unroll
  for (int t = 0; t < TM; t++) {
    const int col = m0 + 16 * t + r16;
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const int row = n0 + d_row(q, v);
      if (row < N && col < M) {
        double x = acc[t][v];
        if (EPI == EPI_BIAS_RELU) x = relu64(x);
        const int64_t o = (int64_t)row * M + col;
        if (C) C[o] = (float)x;
        if (C64) C64[o] = x;
      }
    }
  }
}

}  // namespace tc355
