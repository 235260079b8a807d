// Transposed matmul (Section 7, listing tmm / tbmm) on the int8 matrix core, for
// 128 rows of X, a reduction that is a multiple of 64 and a multiple of 64 rows
// of Y -- the paper's largest tmm, (M,K,N) = (128,4096,16384):
//
//   Z(b,n,m) = sum_k X(b,n,k) * Y(b,m,k)
//
// Arithmetic as in the int8 grouped convolution (gconv_i8.hpp): operands become
// 32-bit fixed-point numbers relative to the largest magnitude of their block,
// four signed 8-bit digits each, and the 10 digit products with k + l >= 3 are
// summed exactly in int32 by v_mfma_i32_16x16x64_i8.  A block here is 64
// consecutive k of one matrix row: the reduction is walked in blocks of 64 (one
// MFMA step), every row of X and of Y gets its own scale in every block, and
// the block's integer sums are scaled back and added up in fp64 (one fp64
// fused multiply-add per output and block), so the only roundings are the
// operands' quantisation (2^-32 of the block maximum), the dropped digit pairs
// (the same size) and K/64 fp64 additions; the result is rounded to fp32 once.
//
// One workgroup of 8 wavefronts = all 128 rows of X against 64 rows of Y.
// Both operands are sliced by the workgroup that uses them (no workspace): X is
// sliced again by every workgroup, which is what bounds this kernel -- about
// twice the vector-ALU work of its matrix work.  Per block of 64 k a thread
// owns 16 elements of one X row (four lanes per row) and 8 of one Y row (eight
// lanes per row): row maximum across those lanes (data-parallel primitives),
// scale = S / max by a reciprocal and two Newton steps, digits, and one 16-byte
// (8-byte) LDS write per digit plane.  The position of a k inside the 64 slots
// of the instruction is free as long as X and Y agree; lanes fetch 16-byte
// pieces so that four (eight) neighbours read one contiguous 256-byte row piece
// and still own 16 (8) consecutive slots.  Digit planes are double-buffered in
// LDS ([plane][row][64 + 16 bytes]); the fp32 blocks are fetched two blocks
// ahead into registers; one barrier per block.  Wavefront w contracts the 16
// rows of Y number w % 4 against 64 rows of X (half w / 4): 4 tiles x 10 MFMAs
// per block.  MFMA rows = rows of Y, columns = rows of X, so a lane ends up with
// four consecutive m of one n: one 16-byte store.
//
// A row of X (of Y) that holds Inf or NaN gives NaN in every output of that row
// (column), as the exact sum would except where an Inf meets only zeros or Infs
// of one sign.
#pragma once
#include "gconv_i8.hpp"

namespace tc355 {

struct GemmI8Args {
  const float* X;  // [B][128][K]
  const float* Y;  // [B][M][K]
  float* Z;        // [B][128][M]
  int M, K;
};

constexpr int GI8_TN = 128, GI8_TM = 64, GI8_KB = 64, GI8_THREADS = 512;
constexpr int GI8_ROWS = GI8_TN + GI8_TM;               // rows staged per block: X rows, then Y rows
constexpr int GI8_RS = GI8_KB + 16;                     // bytes between rows of a digit plane: 16 rows -> 16 bank groups
constexpr int GI8_PLANE = GI8_ROWS * GI8_RS;
constexpr int GI8_BUF = 4 * GI8_PLANE + GI8_ROWS * 8;   // four digit planes and the rows' inverse scales (fp64)
constexpr int GI8_LDS_BYTES = 2 * GI8_BUF;              // 125,952 bytes: one workgroup per compute unit
static_assert(GI8_BUF % 16 == 0 && (4 * GI8_PLANE) % 16 == 0, "16-byte LDS accesses");

// S / max and max / S for a block with largest magnitude bits mbits: the reciprocal by two Newton steps on the
// hardware estimate (relative error far below the 2^-31 that keeps rint(max * scale) inside four digits).
__device__ __forceinline__ void gi8_scales(unsigned mbits, double& scale, double& inverse) {
  const double inv = (double)__uint_as_float(mbits) * I8_INV_FULL;
  double r = __builtin_amdgcn_rcp(inv);
  r = __builtin_fma(__builtin_fma(-inv, r, 1.0), r, r);
  r = __builtin_fma(__builtin_fma(-inv, r, 1.0), r, r);
  scale = mbits ? r : 1.0;
  inverse = i8_nonfinite(mbits) ? __longlong_as_double(0x7ff8000000000000ll) : inv;
}

__global__ __launch_bounds__(GI8_THREADS, 1) void gemm_i8_kernel(GemmI8Args p) {
  extern __shared__ __attribute__((aligned(16))) char gi8g_lds[];
  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int M = p.M, K = p.K, nb = K / GI8_KB;
  const int m0 = blockIdx.x * GI8_TM;
  const int64_t b = blockIdx.y;
  const float* X = p.X + b * (int64_t)GI8_TN * K;
  const float* Y = p.Y + (b * M + m0) * (int64_t)K;
  float* Z = p.Z + b * (int64_t)GI8_TN * M;

  // ---- staging role: 16 slots of X row tid / 4 (slots 16 cx ..), 8 slots of Y row tid / 8 (slots 8 cy ..).
  // Slot 16 c + 4 j + e holds k = 16 j + 4 c + e: the j-th 16-byte piece of lane c.
  const int xrow = tid >> 2, cx = tid & 3;
  const int yrow = tid >> 3, cy = tid & 7;
  const float* xsrc = X + (int64_t)xrow * K + 4 * cx;
  const float* ysrc = Y + (int64_t)yrow * K + 32 * (cy & 1) + 4 * (cy >> 1);
  struct Raw {
    f4 x[4];
    f4 y[2];
  };
  auto fetch = [&](Raw& r, int blk) {
    const float* xs = xsrc + blk * GI8_KB;
    const float* ys = ysrc + blk * GI8_KB;
#pragma unroll
    for (int j = 0; j < 4; j++) r.x[j] = *reinterpret_cast<const f4*>(xs + 16 * j);
#pragma unroll
    for (int j = 0; j < 2; j++) r.y[j] = *reinterpret_cast<const f4*>(ys + 16 * j);
  };
  auto absmax4 = [](const f4& v, unsigned m) {
    const unsigned a0 = __float_as_uint(v.x) & 0x7fffffffu, a1 = __float_as_uint(v.y) & 0x7fffffffu;
    const unsigned a2 = __float_as_uint(v.z) & 0x7fffffffu, a3 = __float_as_uint(v.w) & 0x7fffffffu;
    return i8_max3(i8_max3(a0, a1, a2), a3, m);
  };
  auto digits4 = [](const f4& v, double scale, int (&y)[4]) {
    int d[4];
    d[0] = i8_fixed<0x00808080>(v.x, scale) ^ 0x00808080;  // byte k = digit k
    d[1] = i8_fixed<0x00808080>(v.y, scale) ^ 0x00808080;
    d[2] = i8_fixed<0x00808080>(v.z, scale) ^ 0x00808080;
    d[3] = i8_fixed<0x00808080>(v.w, scale) ^ 0x00808080;
    i8_transpose4(d, y);
  };
  auto slice = [&](const Raw& r, int buf) {
    char* base = gi8g_lds + buf * GI8_BUF;
    double* invs = reinterpret_cast<double*>(base + 4 * GI8_PLANE);
    {  // X: 16 elements, row shared by the 4 lanes of a quad
      unsigned m = 0;
#pragma unroll
      for (int j = 0; j < 4; j++) m = absmax4(r.x[j], m);
      int v = (int)m;
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
      double scale, inverse;
      gi8_scales((unsigned)v, scale, inverse);
      int y[4][4];
#pragma unroll
      for (int j = 0; j < 4; j++) digits4(r.x[j], scale, y[j]);
      char* dst = base + xrow * GI8_RS + 16 * cx;
#pragma unroll
      for (int k = 0; k < 4; k++) {
        i4 rec;
        rec.x = y[0][k]; rec.y = y[1][k]; rec.z = y[2][k]; rec.w = y[3][k];
        *reinterpret_cast<i4*>(dst + k * GI8_PLANE) = rec;
      }
      if (cx == 0) invs[xrow] = inverse;
    }
    {  // Y: 8 elements, row shared by 8 lanes
      unsigned m = absmax4(r.y[0], 0u);
      m = absmax4(r.y[1], m);
      int v = (int)m;
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));  // row_half_mirror: the other quad
      double scale, inverse;
      gi8_scales((unsigned)v, scale, inverse);
      int y[2][4];
#pragma unroll
      for (int j = 0; j < 2; j++) digits4(r.y[j], scale, y[j]);
      char* dst = base + (GI8_TN + yrow) * GI8_RS + 8 * cy;
#pragma unroll
      for (int k = 0; k < 4; k++) {
        int2 rec;
        rec.x = y[0][k]; rec.y = y[1][k];
        *reinterpret_cast<int2*>(dst + k * GI8_PLANE) = rec;
      }
      if (cy == 0) invs[GI8_TN + yrow] = inverse * 16777216.0;  // 2^24: the weight of the lowest kept diagonal
    }
  };

  // ---- contraction role: rows of Y 16 mt .., rows of X 64 nh .. (four tiles)
  const int mt = wave & 3, nh = wave >> 2;
  double acc[4][4];
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int v = 0; v < 4; v++) acc[j][v] = 0.0;
  auto contract = [&](int buf) {
    const char* base = gi8g_lds + buf * GI8_BUF;
    const double* invs = reinterpret_cast<const double*>(base + 4 * GI8_PLANE);
    const char* ya = base + (GI8_TN + 16 * mt + r16) * GI8_RS + 16 * q;
    i4 a[4];
#pragma unroll
    for (int k = 0; k < 4; k++) a[k] = *reinterpret_cast<const i4*>(ya + k * GI8_PLANE);
    double fy[4];
#pragma unroll
    for (int v = 0; v < 4; v++) fy[v] = invs[GI8_TN + 16 * mt + 4 * q + v];
    constexpr int PK[10] = {3, 3, 3, 3, 2, 2, 2, 1, 1, 0};
    constexpr int PL[10] = {3, 2, 1, 0, 3, 2, 1, 3, 2, 3};
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int xr = 64 * nh + 16 * j + r16;
      const char* xb = base + xr * GI8_RS + 16 * q;
      i4 bq[4];
#pragma unroll
      for (int l = 0; l < 4; l++) bq[l] = *reinterpret_cast<const i4*>(xb + l * GI8_PLANE);
      const double fx = invs[xr];
      i4 d[4];  // d[i]: diagonal k + l = 3 + i
#pragma unroll
      for (int i = 0; i < 4; i++) d[i] = i4{0, 0, 0, 0};
#pragma unroll
      for (int pr = 0; pr < 10; pr++) d[PK[pr] + PL[pr] - 3] = mfma_i8(a[PK[pr]], bq[PL[pr]], d[PK[pr] + PL[pr] - 3]);
#pragma unroll
      for (int v = 0; v < 4; v++) {
        const int hi = d[3][v] * 256 + d[2][v], lo = d[1][v] * 256 + d[0][v];  // < 2^29: 64 terms of 2^14 per pair
        const double rr = __builtin_fma((double)hi, 65536.0, (double)lo);
        acc[j][v] = __builtin_fma(rr, fy[v] * fx, acc[j][v]);
      }
    }
  };

  Raw r0, r1;
  fetch(r0, 0);
  fetch(r1, min(1, nb - 1));
  slice(r0, 0);
  fetch(r0, min(2, nb - 1));
  __syncthreads();
  for (int t = 0; t < nb; t += 2) {
    // block t is in buffer 0; r1 holds block t + 1, r0 block t + 2 (indices past the end re-read the last block)
    if (t + 1 < nb) slice(r1, 1);
    fetch(r1, min(t + 3, nb - 1));
    contract(0);
    __syncthreads();
    if (t + 1 >= nb) break;
    if (t + 2 < nb) slice(r0, 0);
    fetch(r0, min(t + 4, nb - 1));
    contract(1);
    __syncthreads();
  }

#pragma unroll
  for (int j = 0; j < 4; j++) {
    f4 o;
    o.x = (float)acc[j][0]; o.y = (float)acc[j][1]; o.z = (float)acc[j][2]; o.w = (float)acc[j][3];
    *reinterpret_cast<f4*>(Z + (int64_t)(64 * nh + 16 * j + r16) * M + m0 + 16 * mt + 4 * q) = o;
  }
}

}  // namespace tc355
