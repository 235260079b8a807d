// Lookup-table sums (Section 7, production model; appendix listing 2LUT):
//   O_t(i,j) +=! LUT_t(Idx_t(i,k), j)          for every table t of the call
// A pure gather: B*L rows of D floats out of a table of E rows (the paper's
// sizes: E = 10^7, D = 64, L = 50, B = 128: 1.6 MB gathered out of 2.56 GB),
// summed per output row.  Nothing here is a contraction; what matters is that
// every load of a row is in flight at once instead of one after the other
// (the paper's two-stage loading serves the same end): a thread first reads
// all its indices (one round trip), then all its table rows (a second one).
//
// One workgroup per (table, output row, block of columns).  A row of D floats
// is read as D/V units of V floats (V = 4: 16-byte loads); the 256 threads are
// `slots` groups of `cpw` threads: thread (slot s, column unit u) sums the
// lookups k = s, s + slots, ... of its unit in fp64, and the slots are combined
// through LDS in slot order.  At D = 64 that is 16 slots of 16 threads, at most
// four lookups per thread.  Every sum is exact up to the final rounding to
// fp32 (fp64 holds the sum of 2^29 floats of equal exponent range exactly
// enough: the error is far below one fp32 rounding).
//
// An index outside [0, E) has no meaning in the comprehension: nothing is read
// for it, and the whole output row is NaN.
#pragma once
#include "tc355_device.hpp"

namespace tc355 {

constexpr int LUT_MAX_TABLES = 8;
constexpr int LUT_NB = 4;  // lookups in flight per thread and round

struct LutArgs {
  const float* LUT[LUT_MAX_TABLES];  // [E][D]
  const int* Idx[LUT_MAX_TABLES];    // [B][L]
  float* O[LUT_MAX_TABLES];          // [B][D]
  long long E[LUT_MAX_TABLES];
  int L[LUT_MAX_TABLES];
  int D, B;
  int cpw;     // column units per workgroup: a power of two, <= 256
  int blocks;  // column blocks per row: ceil(D / V / cpw)
};

template <int V>
__global__ __launch_bounds__(WG_THREADS) void lut_sum_kernel(LutArgs p) {
  __shared__ double part[WG_THREADS * V];
  const int tid = threadIdx.x;
  const int cpw = p.cpw, slots = WG_THREADS / cpw;
  const int ul = tid & (cpw - 1), s = tid / cpw;
  int job = blockIdx.x;
  const int cb = job % p.blocks; job /= p.blocks;
  const int i = job % p.B;
  const int t = job / p.B;
  const int units = p.D / V;
  const int u = cb * cpw + ul;
  const bool ucol = u < units;
  const int L = p.L[t];
  const long long E = p.E[t];
  const int* idx = p.Idx[t] + (int64_t)i * L;
  const float* tab = p.LUT[t] + (int64_t)u * V;

  double acc[V];
#pragma unroll
  for (int e = 0; e < V; e++) acc[e] = 0.0;
  bool bad = false;
  for (int k0 = s; k0 < L; k0 += slots * LUT_NB) {
    int row[LUT_NB];
    bool ok[LUT_NB];
    // stage 1: the indices of this round
#pragma unroll
    for (int j = 0; j < LUT_NB; j++) {
      const int k = k0 + j * slots;
      ok[j] = k < L;
      row[j] = ok[j] ? idx[k] : 0;
    }
#pragma unroll
    for (int j = 0; j < LUT_NB; j++) {
      const bool inside = row[j] >= 0 && (long long)row[j] < E;
      bad = bad || (ok[j] && !inside);
      ok[j] = ok[j] && inside && ucol;
    }
    // stage 2: the table rows, all requested before the first is used
    Vec<float, V> val[LUT_NB];
#pragma unroll
    for (int j = 0; j < LUT_NB; j++) {
      if (ok[j]) val[j] = load_vec<float, V>(tab + (int64_t)row[j] * p.D);
    }
#pragma unroll
    for (int j = 0; j < LUT_NB; j++) {
      if (ok[j]) {
#pragma unroll
        for (int e = 0; e < V; e++) acc[e] += (double)val[j].e[e];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < V; e++) part[(s * cpw + ul) * V + e] = acc[e];
  const int any_bad = __syncthreads_or(bad ? 1 : 0);
  if (s == 0 && ucol) {
    float* out = p.O[t] + (int64_t)i * p.D + (int64_t)u * V;
    float r[V];
#pragma unroll
    for (int e = 0; e < V; e++) {
      double x = 0.0;
      for (int ss = 0; ss < slots; ss++) x += part[(ss * cpw + ul) * V + e];
      r[e] = any_bad ? __builtin_nanf("") : (float)x;
    }
    if constexpr (V == 4) {
      *reinterpret_cast<f4*>(out) = f4{r[0], r[1], r[2], r[3]};
    } else {
#pragma unroll
      for (int e = 0; e < V; e++) out[e] = r[e];
    }
  }
}

}  // namespace tc355
