// Transposed matmul (Section 7, listing tmm / tbmm) on the int8 matrix core, for
// a multiple of 128 rows of X, a reduction that is a multiple of 4 (at least 256;
// the last block of 128 is filled with zeros) and a multiple of 64 rows of Y --
// the paper's largest tmm, (M,K,N) = (128,4096,16384):
//
//   Z(b,n,m) = sum_k X(b,n,k) * Y(b,m,k)
//
// Arithmetic as in the int8 grouped convolution (gconv_i8.hpp): operands become
// 32-bit fixed-point numbers relative to the largest magnitude of their block,
// four signed 8-bit digits each, and the 10 digit products with k + l >= 3 are
// summed exactly in int32 by v_mfma_i32_16x16x64_i8.  A block here is 128
// consecutive k of one matrix row (two MFMA steps): every row of X and of Y
// gets its own scale in every block, and the block's integer sums are scaled
// back and added up in fp64 (one fp64 fused multiply-add per output and
// block), so the only roundings are the operands' quantisation (2^-32 of the
// block maximum), the dropped digit pairs (the same size) and K/128 fp64
// additions; the result is rounded to fp32 once.
//
// One workgroup of 8 wavefronts = 128 rows of X against 64 rows of Y.
// Without a workspace both operands are sliced by the workgroup that uses them:
// X is sliced again by every workgroup, and slicing plus the per-block scaling
// of the sums is about 475 vector-ALU instructions per wavefront and block
// beside its 104 MFMAs (13 digit products).  With a workspace (PRE = true) X is
// sliced ONCE by gemm_i8_slice_x_kernel, which runs the X half of the slicing
// code and writes the digit records and the rows' inverse scales to global
// memory in exactly the order in which this kernel's threads pick them up (one
// 16-byte load per record, 8 KiB of consecutive addresses per instruction of
// the workgroup): 184 of the vector instructions per wavefront and block go.  On this chip the vector ALU and the matrix core of a SIMD do
// not work at the same time (the time of this kernel is the sum of its two
// halves whatever their order or interleaving), so the kernel is bound by that
// sum; blocks of 128 instead of 64 halve the per-block scaling work.
// Per block a thread owns 32 elements of one X row (four lanes per row) and 16
// of one Y row (eight lanes per row): row maximum across those lanes
// (data-parallel primitives), scale = S / max by a reciprocal and two Newton
// steps, digits, and 16-byte (8-byte) LDS writes per digit plane.  The position
// of a k inside the 64 slots of an MFMA step is free as long as X and Y agree;
// lanes fetch 16-byte pieces so that four (eight) neighbours read one
// contiguous 256-byte row piece and still own 16 (8) consecutive slots.  The
// digit planes sit in LDS once ([plane][row][128 + 32 bytes]: a row stride
// that the operand reads take without bank conflicts); the next fp32 block is
// fetched into registers while the current one is contracted; two barriers
// per block.
// Wavefront w contracts the 16 rows of Y number w % 4 against 64 rows of X
// (half w / 4): 4 tiles x 20 MFMAs per block.  MFMA rows = rows of Y, columns =
// rows of X, so a lane ends up with four consecutive m of one n: one 16-byte
// store.
//
// A row of X (of Y) that holds Inf or NaN gives NaN in every output of that row
// (column), as the exact sum would except where an Inf meets only zeros or Infs
// of one sign.
#pragma once
#include "gconv_i8.hpp"

namespace tc355 {

struct GemmI8Args {
  const float* X;  // [B][N][K], N = 128 * gridDim.z
  const float* Y;  // [B][M][K]
  float* Z;        // [B][N][M]
  int M, K;
  // X sliced beforehand (PRE = true): per block of 128 rows and block of 128 k, 8 record groups (MFMA step s, digit
  // plane k) of 512 records of 16 bytes, record t being what thread t of the contracting workgroup stages; then
  // the 128 inverse scales of the block (fp64)
  const i4* Xd;        // [B * N / 128][K / 128][2][4][512]
  const double* Xinv;  // [B * N / 128][K / 128][128]
};
// bytes of pre-sliced X per block of 128 rows x 128 k
constexpr int64_t GI8_XD_BYTES = 2 * 4 * 512 * 16, GI8_XINV_BYTES = 128 * 8;

constexpr int GI8_TN = 128, GI8_TM = 64, GI8_KB = 128, GI8_THREADS = 512;
constexpr int GI8_STEPS = GI8_KB / 64;                  // MFMA steps (64 reduction slots each) per block
constexpr int GI8_ROWS = GI8_TN + GI8_TM;               // rows staged per block: X rows, then Y rows
// Bytes between rows of a digit plane: 10 chunks of 16 bytes.  Measured on this chip with the MFMA operand pattern
// (lane (r16, q) reads chunk q of row r16): row strides of 6 and 10 chunks read at full speed (4.5 clocks per
// wavefront), strides of 4, 5, 9 and 17 chunks and several XOR permutations of unpadded rows take twice as long.
constexpr int GI8_RS = GI8_KB + 32;
constexpr int GI8_PLANE = GI8_ROWS * GI8_RS;
constexpr int GI8_LDS_BYTES = 4 * GI8_PLANE + GI8_ROWS * 8;  // four digit planes and the rows' inverse scales (fp64): 124,416 bytes
static_assert(GI8_LDS_BYTES % 16 == 0 && (4 * GI8_PLANE) % 16 == 0, "16-byte LDS accesses");
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

// MIND: the lowest digit diagonal k + l that is kept: 2 (13 products: what the library uses unless told that 10
// will do) or 3 (10 products).
// The digits of four elements, transposed: y[k] = digit k of the four (the offset that makes the digits signed is
// removed after the transposition: three instructions instead of four).
__device__ __forceinline__ void gi8_digits4(const f4& v, double scale, int (&y)[4]) {
  int d[4];
  d[0] = i8_fixed<0x00808080>(v.x, scale);
  d[1] = i8_fixed<0x00808080>(v.y, scale);
  d[2] = i8_fixed<0x00808080>(v.z, scale);
  d[3] = i8_fixed<0x00808080>(v.w, scale);
  i8_transpose4(d, y);
  y[0] ^= 0x80808080; y[1] ^= 0x80808080; y[2] ^= 0x80808080;
}
// Largest magnitude without clearing sign bits: as signed integers the non-negative floats order by magnitude
// and lie above every negative one; as unsigned integers the negative ones order by magnitude and lie above
// every non-negative one.  One signed and one unsigned three-way maximum per two elements, merged at the end.
__device__ __forceinline__ void gi8_absmax4(const f4& v, int& smax, unsigned& umax) {
  const int s0 = __float_as_int(v.x), s1 = __float_as_int(v.y), s2 = __float_as_int(v.z), s3 = __float_as_int(v.w);
  smax = i8_max3(i8_max3(s0, s1, s2), s3, smax);
  umax = i8_max3(i8_max3((unsigned)s0, (unsigned)s1, (unsigned)s2), (unsigned)s3, umax);
}
__device__ __forceinline__ int gi8_magnitude(int smax, unsigned umax) { return max(max(smax, 0), (int)(umax & 0x7fffffffu)); }

// X sliced once: one workgroup per (block of 128 k, block of 128 rows), thread t = (row t / 4, chunk t % 4) exactly
// as in the contracting kernel, which later reads record t of every group with one 16-byte load.
__global__ __launch_bounds__(GI8_THREADS, 1) void gemm_i8_slice_x_kernel(const float* X, int K, i4* Xd, double* Xinv) {
  const int tid = threadIdx.x, blk = blockIdx.x, nb = (K + GI8_KB - 1) / GI8_KB;
  const int64_t rb = blockIdx.y;
  const int xrow = tid >> 2, cx = tid & 3;
  const float* xs = X + (rb * GI8_TN + xrow) * (int64_t)K + (int64_t)blk * GI8_KB + 4 * cx;
  f4 rx[GI8_STEPS][4];
#pragma unroll
  for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
    for (int j = 0; j < 4; j++) {  // K is a multiple of 4: whole pieces; past the end of the reduction: zeros
      const bool in = blk * GI8_KB + 64 * s + 16 * j + 4 * cx < K;
      rx[s][j] = in ? *reinterpret_cast<const f4*>(xs + 64 * s + 16 * j) : f4{0.f, 0.f, 0.f, 0.f};
    }
  int sm = 0;
  unsigned um = 0;
#pragma unroll
  for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
    for (int j = 0; j < 4; j++) gi8_absmax4(rx[s][j], sm, um);
  int v = gi8_magnitude(sm, um);
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
  double scale, inverse;
  gi8_scales((unsigned)v, scale, inverse);
  i4* dst = Xd + (rb * nb + blk) * (int64_t)(GI8_STEPS * 4 * GI8_THREADS) + tid;
#pragma unroll
  for (int s = 0; s < GI8_STEPS; s++) {
    int y[4][4];
#pragma unroll
    for (int j = 0; j < 4; j++) gi8_digits4(rx[s][j], scale, y[j]);
#pragma unroll
    for (int k = 0; k < 4; k++) {
      i4 rec;
      rec.x = y[0][k]; rec.y = y[1][k]; rec.z = y[2][k]; rec.w = y[3][k];
      dst[(s * 4 + k) * GI8_THREADS] = rec;
    }
  }
  if (cx == 0) Xinv[(rb * nb + blk) * GI8_TN + xrow] = inverse;
}

// PRE: X arrives sliced (Xd, Xinv) instead of as fp32.
template <int MIND = 2, bool PRE = false>
__global__ __launch_bounds__(GI8_THREADS, 1) void gemm_i8_kernel(GemmI8Args p) {
  static_assert(MIND == 2 || MIND == 3, "13 or 10 digit products");
  extern __shared__ __attribute__((aligned(16))) char gi8g_lds[];
  const int tid = threadIdx.x;
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  const int r16 = lane & 15, q = lane >> 4;
  const int M = p.M, K = p.K, nb = (K + GI8_KB - 1) / GI8_KB;  // the last block of a K that is no multiple of 128 is filled with zeros
  const int m0 = blockIdx.x * GI8_TM;
  const int64_t b = blockIdx.y;
  const int64_t n0 = (b * gridDim.z + blockIdx.z) * GI8_TN;  // first row of this workgroup's 128 in [B * N]
  const float* X = p.X + n0 * K;
  const float* Y = p.Y + (b * M + m0) * (int64_t)K;
  float* Z = p.Z + n0 * M;
  double* invs = reinterpret_cast<double*>(gi8g_lds + 4 * GI8_PLANE);

  // ---- staging role: 16 slots per MFMA step of X row tid / 4 (chunk cx of the step), 8 slots per step of Y row
  // tid / 8 (half hy of chunk cyc).  Slot 16 c + 4 j + e of step s holds k = 64 s + 16 j + 4 c + e: the j-th
  // 16-byte piece of lane c in that step's 256 bytes of the row.
  const int xrow = tid >> 2, cx = tid & 3;
  const int yrow = tid >> 3, cyc = (tid & 7) >> 1, hy = tid & 1;
  const float* xsrc = X + (int64_t)xrow * K + 4 * cx;
  const float* ysrc = Y + (int64_t)yrow * K + 32 * hy + 4 * cyc;
  f4 rx[GI8_STEPS][4], ry[GI8_STEPS][2];
  i4 xd[GI8_STEPS][4];  // PRE: this thread's digit records of the block
  double xinv = 0.0;    // PRE: inverse scale of row xrow in the block
  const int64_t rb = b * gridDim.z + blockIdx.z;  // block of 128 rows of X
  auto fetch = [&](int blk) {
    const float* ys = ysrc + blk * GI8_KB;
    const bool whole = blk * GI8_KB + GI8_KB <= K;  // K is a multiple of 4: 16-byte pieces are inside or outside as a whole
    if constexpr (PRE) {
      const i4* xr = p.Xd + (rb * nb + blk) * (int64_t)(GI8_STEPS * 4 * GI8_THREADS) + tid;
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
        for (int k = 0; k < 4; k++) xd[s][k] = xr[(s * 4 + k) * GI8_THREADS];
      xinv = p.Xinv[(rb * nb + blk) * GI8_TN + xrow];
    } else {
      const float* xs = xsrc + blk * GI8_KB;
      if (whole) {
#pragma unroll
        for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
          for (int j = 0; j < 4; j++) rx[s][j] = *reinterpret_cast<const f4*>(xs + 64 * s + 16 * j);
      } else {
#pragma unroll
        for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
          for (int j = 0; j < 4; j++) {
            const bool in = blk * GI8_KB + 64 * s + 16 * j + 4 * cx < K;
            rx[s][j] = in ? *reinterpret_cast<const f4*>(xs + 64 * s + 16 * j) : f4{0.f, 0.f, 0.f, 0.f};
          }
      }
    }
    if (whole) {
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
        for (int j = 0; j < 2; j++) ry[s][j] = *reinterpret_cast<const f4*>(ys + 64 * s + 16 * j);
    } else {
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
          const bool in = blk * GI8_KB + 64 * s + 16 * j + 32 * hy + 4 * cyc < K;
          ry[s][j] = in ? *reinterpret_cast<const f4*>(ys + 64 * s + 16 * j) : f4{0.f, 0.f, 0.f, 0.f};
        }
    }
  };
  auto slice = [&]() {
    if constexpr (PRE) {  // X: the records as they came
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++) {
        char* dst = gi8g_lds + xrow * GI8_RS + 16 * (4 * s + cx);
#pragma unroll
        for (int k = 0; k < 4; k++) *reinterpret_cast<i4*>(dst + k * GI8_PLANE) = xd[s][k];
      }
      invs[xrow] = xinv;
    } else {  // X: 16 elements per step, row shared by the 4 lanes of a quad
      int sm = 0;
      unsigned um = 0;
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++)
#pragma unroll
        for (int j = 0; j < 4; j++) gi8_absmax4(rx[s][j], sm, um);
      int v = gi8_magnitude(sm, um);
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
      double scale, inverse;
      gi8_scales((unsigned)v, scale, inverse);
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++) {
        int y[4][4];
#pragma unroll
        for (int j = 0; j < 4; j++) gi8_digits4(rx[s][j], scale, y[j]);
        char* dst = gi8g_lds + xrow * GI8_RS + 16 * (4 * s + cx);
#pragma unroll
        for (int k = 0; k < 4; k++) {
          i4 rec;
          rec.x = y[0][k]; rec.y = y[1][k]; rec.z = y[2][k]; rec.w = y[3][k];
          *reinterpret_cast<i4*>(dst + k * GI8_PLANE) = rec;
        }
      }
      invs[xrow] = inverse;  // the four lanes of the row write the same value: no branch in the step
    }
    {  // Y: 8 elements per step, row shared by 8 lanes
      int sm = 0;
      unsigned um = 0;
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++) {
        gi8_absmax4(ry[s][0], sm, um);
        gi8_absmax4(ry[s][1], sm, um);
      }
      int v = gi8_magnitude(sm, um);
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
      v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));  // row_half_mirror: the other quad
      double scale, inverse;
      gi8_scales((unsigned)v, scale, inverse);
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++) {
        int y[2][4];
#pragma unroll
        for (int j = 0; j < 2; j++) gi8_digits4(ry[s][j], scale, y[j]);
        char* dst = gi8g_lds + (GI8_TN + yrow) * GI8_RS + 16 * (4 * s + cyc) + 8 * hy;
#pragma unroll
        for (int k = 0; k < 4; k++) {
          int2 rec;
          rec.x = y[0][k]; rec.y = y[1][k];
          *reinterpret_cast<int2*>(dst + k * GI8_PLANE) = rec;
        }
      }
      invs[GI8_TN + yrow] = inverse * 16777216.0;  // 2^24: the weight of the lowest kept diagonal
    }
  };

  // ---- contraction role: rows of Y 16 mt .., rows of X 64 nh .. (four tiles)
  const int mt = wave & 3, nh = wave >> 2;
  double acc[4][4];
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int v = 0; v < 4; v++) acc[j][v] = 0.0;
  auto contract = [&]() {
    i4 a[GI8_STEPS][4];
#pragma unroll
    for (int s = 0; s < GI8_STEPS; s++) {
      const char* ya = gi8g_lds + (GI8_TN + 16 * mt + r16) * GI8_RS + 16 * (4 * s + q);
#pragma unroll
      for (int k = 0; k < 4; k++) a[s][k] = *reinterpret_cast<const i4*>(ya + k * GI8_PLANE);
    }
    double fy[4];
#pragma unroll
    for (int v = 0; v < 4; v++) fy[v] = invs[GI8_TN + 16 * mt + 4 * q + v];
    // order: no two consecutive products on one diagonal
    constexpr int ND = 7 - MIND, NP = MIND == 3 ? 10 : 13;
    constexpr int PK[13] = {3, 2, 3, 3, 2, 1, 2, 1, 0, 3, 2, 1, 0};  // the last three: the diagonal k + l = 2
    constexpr int PL[13] = {0, 1, 1, 2, 2, 2, 3, 3, 3, 3, 0, 1, 2};
    i4 d[2][ND];  // d[.][i]: diagonal k + l = MIND + i; two sets, so that a tile's MFMAs run under the previous tile's epilogue
    double fx[2];
    auto mma = [&](int j, i4 (&dd)[ND], double& fxj) {
      const int xr = 64 * nh + 16 * j + r16;
#pragma unroll
      for (int i = 0; i < ND; i++) dd[i] = i4{0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < GI8_STEPS; s++) {
        const char* xb = gi8g_lds + xr * GI8_RS + 16 * (4 * s + q);
        i4 bq[4];
#pragma unroll
        for (int l = 0; l < 4; l++) bq[l] = *reinterpret_cast<const i4*>(xb + l * GI8_PLANE);
#pragma unroll
        for (int pr = 0; pr < NP; pr++)
          dd[PK[pr] + PL[pr] - MIND] = mfma_i8(a[s][PK[pr]], bq[PL[pr]], dd[PK[pr] + PL[pr] - MIND]);
      }
      fxj = invs[xr];
    };
    auto epilogue = [&](int j, const i4 (&dd)[ND], double fxj) {
#pragma unroll
      for (int v = 0; v < 4; v++) {
        // 128 terms of at most 2^14 per digit pair: 2^21 x 256 + 2 x 2^21 and 3 x 2^21 x 256 + 4 x 2^21, below 2^31
        const int hi = dd[ND - 1][v] * 256 + dd[ND - 2][v], lo = dd[ND - 3][v] * 256 + dd[ND - 4][v];
        double rr = __builtin_fma((double)hi, 65536.0, (double)lo);
        if constexpr (MIND == 2) rr = __builtin_fma((double)dd[0][v], 0.00390625, rr);
        acc[j][v] = __builtin_fma(rr, fy[v] * fxj, acc[j][v]);
      }
    };
    mma(0, d[0], fx[0]);
    mma(1, d[1], fx[1]);
    epilogue(0, d[0], fx[0]);
    mma(2, d[0], fx[0]);
    epilogue(1, d[1], fx[1]);
    mma(3, d[1], fx[1]);
    epilogue(2, d[0], fx[0]);
    epilogue(3, d[1], fx[1]);
  };

  // One block: stage it from the registers, refill them with the next block (a whole block of time ahead of its
  // use; past the end the last block is read again), contract.  The vector ALU and the matrix core of a SIMD do
  // not run at the same time on this chip, so nothing is lost by not overlapping the two halves, and a single
  // LDS buffer makes room for blocks of 128.
  fetch(0);
  for (int t = 0; t < nb; t++) {
    slice();
    // with 13 digit products the loads are issued behind the barrier, where their address work runs under the first
    // tile's MFMAs (-3 .. -4 %); with 10 that order measured 2 % slower
    if constexpr (MIND == 3) fetch(min(t + 1, nb - 1));
    __syncthreads();
    if constexpr (MIND == 2) fetch(min(t + 1, nb - 1));
    contract();
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
