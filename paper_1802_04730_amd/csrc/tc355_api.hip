// Host side of libtc355: argument validation, kernel selection and launches
// for the entry points declared in include/tc355.h.
#include "../../include/tc355.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <random>
#include <type_traits>

#include "gconv_band.hpp"
#include "gconv_i8.hpp"
#include "gconv_i8_c32.hpp"
#include "gemm_i8.hpp"
#include "gconv_i8_small.hpp"
#include "gconv_lds.hpp"
#include "gconv_quad.hpp"
#include "gconv_tiny.hpp"
#include "gconv_wave.hpp"
#include "gemm_tile.hpp"
#include "gemm_wave.hpp"
#include "kron_lds.hpp"
#include "kron_wave.hpp"
#include "lut_sum.hpp"
#include "mlp_fused.hpp"
#include "mlp_rows.hpp"
#include "sconv_tile.hpp"
#include "sconv_i8.hpp"
#include "tbmm_lds.hpp"

using namespace tc355;

namespace {

constexpr int64_t kMaxElems = (int64_t)1 << 31;  // per-tensor element limit of the 32-bit in-tile indexing
constexpr int64_t kMaxGrid = 2147483647;

inline bool misaligned(const void* p, size_t a = 16) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// True if the product of the (positive) extents reaches `limit`; never overflows: it stops at the first factor
// that takes the running product there.
inline bool prod_reaches(std::initializer_list<int64_t> factors, int64_t limit) {
  int64_t p = 1;
  for (int64_t f : factors) {
    if (f >= limit || p > limit / f) return true;  // p * f > limit
    p *= f;
    if (p >= limit) return true;
  }
  return false;
}

inline tc_status launch_status() { return hipGetLastError() == hipSuccess ? TC_OK : TC_ERR_LAUNCH; }

// Options of the calling host thread (tc355_set_option) and the kernel family its last call chose (tc355_last_path).
struct ThreadOptions {
  int64_t int8 = TC_INT8_AUTO;
  int64_t mlp_kernel = TC_MLP_AUTO;
  int64_t mlp_spin_limit = 4000000;
};
thread_local ThreadOptions t_opt;
thread_local const char* t_path = "";

inline tc_status took(const char* path, tc_status st) {
  t_path = path;
  return st;
}


// ---- generic wave-level contraction launcher --------------------------------
template <typename TA, int VEC, int EPI>
tc_status launch_gemm_tm(GemmArgs a, int64_t batch, int tm, hipStream_t s) {
  a.tiles_n = (int)ceil_div(a.N, 16);
  a.strips_m = (int)ceil_div(a.M, 16 * tm);
  a.jobs = batch * a.tiles_n * a.strips_m;
  const int64_t grid = ceil_div(a.jobs, WAVES_PER_WG);
  if (grid > kMaxGrid) return TC_ERR_UNSUPPORTED;
  const dim3 g((unsigned)grid), b(WG_THREADS);
  switch (tm) {
    case 1: gemm_nt_wave_kernel<TA, VEC, 1, EPI><<<g, b, 0, s>>>(a); break;
    case 2: gemm_nt_wave_kernel<TA, VEC, 2, EPI><<<g, b, 0, s>>>(a); break;
    case 3: gemm_nt_wave_kernel<TA, VEC, 3, EPI><<<g, b, 0, s>>>(a); break;
    case 4: gemm_nt_wave_kernel<TA, VEC, 4, EPI><<<g, b, 0, s>>>(a); break;
    default: gemm_nt_wave_kernel<TA, VEC, 5, EPI><<<g, b, 0, s>>>(a); break;
  }
  return launch_status();
}

// LDS-tiled kernel for big blocks (64 x 64 output tiles); returns false if it does not apply.
template <typename TA, int EPI>
bool try_gemm_tile(const GemmArgs& a, int64_t batch, hipStream_t s, tc_status* st) {
  if (a.K % 4 != 0 || a.N < 48 || a.M < 48) return false;
  const int64_t tiles = ceil_div(a.N, GT_BM) * ceil_div(a.M, GT_BN);
  if (tiles > kMaxGrid || batch > 65535) return false;
  if (tiles * batch < 128) return false;  // too few blocks to fill the chip: the wave-level kernel spreads wider
  static std::atomic<int> lds_ok{0};  // needs more than the default 64 KiB of dynamic LDS
  if (!lds_ok.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_nt_tile_kernel<TA, EPI>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, GT_LDS_BYTES) != hipSuccess) {
      *st = TC_ERR_LAUNCH;
      return true;
    }
    lds_ok.store(1, std::memory_order_release);
  }
  gemm_nt_tile_kernel<TA, EPI><<<dim3((unsigned)tiles, (unsigned)batch), dim3(WG_THREADS), GT_LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

int device_cus();

// ---- grouped convolution with 4 or 8 channels per group (4x4x4 MFMA blocks), compile-time width --------
template <int C, int F, int KH, int KW, int W, int ROWS, int MINW>
bool try_gconv_quad(const GconvArgs& g, hipStream_t s, tc_status* st) {
  using Gm = GconvQuadGeom<C, F, KH, KW, W, ROWS>;
  if (g.C != C || g.F != F || g.KH != KH || g.KW != KW || g.W != W) return false;
  const int64_t grid = (int64_t)g.N * g.G;
  if (grid > kMaxGrid) return false;
  static std::atomic<int> lds_ok{0};
  if (!lds_ok.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gconv_quad_kernel<C, F, KH, KW, W, ROWS, MINW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Gm::LDS_BYTES) != hipSuccess) {
      *st = TC_ERR_LAUNCH;
      return true;
    }
    lds_ok.store(1, std::memory_order_release);
  }
  GconvQuadArgs a{};
  a.I = g.I; a.W1 = g.W1; a.bias = g.bias; a.O = g.O;
  a.G = g.G; a.H = g.H;
  gconv_quad_kernel<C, F, KH, KW, W, ROWS, MINW><<<dim3((unsigned)grid), dim3(WG_THREADS), Gm::LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

// ---- grouped convolution with a large filter bank on tiny images: the bank stays in registers, images stream ----
template <int C, int F, int KH, int KW, int H, int W>
bool try_gconv_tiny(const GconvArgs& g, hipStream_t s, tc_status* st) {
  using Gm = GconvTinyGeom<C, F, KH, KW, H, W>;
  if (g.C != C || g.F != F || g.KH != KH || g.KW != KW || g.H != H || g.W != W) return false;
  const int cus = device_cus();
  if (cus <= 0) return false;
  // about two workgroups per compute unit: each owns one group and a run of images
  const int64_t nchunks = std::min<int64_t>(g.N, std::max<int64_t>(1, 2 * (int64_t)cus / g.G));
  const int64_t chunk = ceil_div(g.N, nchunks);
  GconvTinyArgs a{};
  a.I = g.I; a.W1 = g.W1; a.bias = g.bias; a.O = g.O;
  a.N = g.N; a.G = g.G;
  a.chunk = (int)chunk;
  a.nchunks = (int)ceil_div(g.N, chunk);
  const int64_t grid = (int64_t)g.G * a.nchunks;
  if (grid > kMaxGrid) return false;
  gconv_tiny_kernel<C, F, KH, KW, H, W><<<dim3((unsigned)grid), dim3(WG_THREADS), Gm::LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

// Split-reduction kernel (the MLP layer body without its epilogue) for one fp32 matrix pair with a long reduction
// and too few 64 x 64 blocks for the kernel above; returns false if it does not apply.
bool try_gemm_splitk(const GemmArgs& a, int64_t batch, hipStream_t s, tc_status* st) {
  if (batch != 1 || a.K % 4 != 0 || a.K < 2 * MLP_KC || !a.C || a.C64) return false;
  // the kernel addresses its operands with 32-bit byte offsets
  if ((int64_t)a.N * a.K * 4 >= (1ll << 32) || (int64_t)a.M * a.K * 4 >= (1ll << 32)) return false;
  const int64_t jobs = ceil_div(a.N, 16) * ceil_div(a.M, 16);
  const int cus = device_cus();
  if (jobs < 64 || cus <= 0) return false;
  static std::atomic<int> lds_ok{0};  // needs more than the default 64 KiB of dynamic LDS
  if (!lds_ok.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_nt_splitk_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, MLP_LDS_BYTES) != hipSuccess) {
      *st = TC_ERR_LAUNCH;
      return true;
    }
    lds_ok.store(1, std::memory_order_release);
  }
  const unsigned nwg = (unsigned)std::min<int64_t>(2 * cus, jobs);
  gemm_nt_splitk_kernel<<<dim3(nwg), dim3(WG_THREADS), MLP_LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

template <typename TA, int EPI>
tc_status launch_gemm(const GemmArgs& a, int64_t batch, int tm, hipStream_t s) {
  tc_status st = TC_OK;
  constexpr bool plain = EPI == EPI_NONE;  // tc_tbmm (else: one MLP layer)
  if (try_gemm_tile<TA, EPI>(a, batch, s, &st)) return took(plain ? "tbmm:tile" : "mlp:layers", st);
  if constexpr (std::is_same<TA, float>::value && EPI == EPI_NONE) {
    if (try_gemm_splitk(a, batch, s, &st)) return took("tbmm:splitk", st);
  }
  t_path = plain ? "tbmm:wave" : "mlp:layers";
  // widest per-lane load that keeps every row start aligned
  if (a.K % 4 == 0) return launch_gemm_tm<TA, 4, EPI>(a, batch, tm, s);
  if (a.K % 2 == 0) return launch_gemm_tm<TA, 2, EPI>(a, batch, tm, s);
  return launch_gemm_tm<TA, 1, EPI>(a, batch, tm, s);
}

// Strip width (in 16-column tiles) that wastes the fewest padded columns; ties go to the wider strip.
int pick_strip(int64_t M, int64_t waves_if_one) {
  const int64_t tiles = ceil_div(M, 16);
  if (tiles <= 5) return (int)tiles;
  if (waves_if_one < 4096) return 1;  // few jobs: favour parallelism over operand reuse
  int best = 1;
  int64_t best_pad = -1;
  for (int tm = 5; tm >= 2; tm--) {
    const int64_t pad = ceil_div(tiles, tm) * tm - tiles;
    if (best_pad < 0 || pad < best_pad) { best = tm; best_pad = pad; }
  }
  return best;
}

size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- tuned grouped convolution: returns false if this instance does not apply -----
template <int C, int F, int KH, int KW, int TP>
bool try_gconv_lds(const GconvArgs& g, hipStream_t s, tc_status* st) {
  if (g.C != C || g.F != F || g.KH != KH || g.KW != KW) return false;
  const int npix = g.OH * g.OW;
  const int rows = gconv_band_rows(64 * TP, g.OW, KH);
  const int PS = gconv_plane_stride(rows * g.W);
  const size_t lds = ((size_t)C * PS + (size_t)(F / 16) * (KH * KW * C / 4) * WAVE) * sizeof(float);
  if (lds > 64 * 1024) return false;
  GconvLdsArgs a{};
  a.I = g.I; a.W1 = g.W1; a.bias = g.bias; a.O = g.O;
  a.G = g.G; a.H = g.H; a.W = g.W; a.OH = g.OH; a.OW = g.OW;
  a.PS = PS;
  a.pblocks = (int)ceil_div(npix, 64 * TP);
  a.ngs = (int64_t)g.N * g.G;
  const int64_t grid = a.ngs * a.pblocks;
  if (grid > kMaxGrid) return false;
  gconv_lds_kernel<C, F, KH, KW, TP><<<dim3((unsigned)grid), dim3(WG_THREADS), lds, s>>>(a);
  *st = launch_status();
  return true;
}

// Number of compute units of the current device (cached per device index).
int device_cus() {
  static std::atomic<int> cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  int cus = cache[dev].load(std::memory_order_relaxed);
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    cache[dev].store(cus, std::memory_order_relaxed);
  }
  return cus;
}

// A fresh 64-bit token per fused-MLP call (low 32 bits never 0): random start, then counting.
unsigned long long next_token() {
  static std::atomic<unsigned long long> tok{[] {
    std::random_device rd;
    unsigned long long t = ((unsigned long long)rd() << 32) ^ rd();
    t ^= (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count();
    return t | 1ull;
  }()};
  unsigned long long t = tok.fetch_add(1, std::memory_order_relaxed);
  while ((t & 0xffffffffull) == 0) t = tok.fetch_add(1, std::memory_order_relaxed);  // low word is what release words carry
  return t;
}

size_t mlp_sync_bytes() { return round256((MLP_SYNC_WORDS + (size_t)(MLP_MAX_LAYERS - 1) * MLP_BAR_WORDS) * sizeof(unsigned)); }

// fp64 copy of one layer's output; whole 16-row tiles (the small-batch kernel keeps it in a tiled layout)
size_t mlp_act_bytes(int64_t batch, int64_t width) {
  return round256((size_t)ceil_div(batch, 16) * 16 * (size_t)width * sizeof(double));
}

// ---- fastest grouped convolution: compile-time width, one workgroup per (image, group) -----
template <int C, int KH, int KW, int W, int ROWS, int MINW>
bool try_gconv_band(const GconvArgs& g, hipStream_t s, tc_status* st) {
  using Gm = GconvBandGeom<C, KH, KW, W, ROWS>;
  if (g.C != C || g.F != Gm::F || g.KH != KH || g.KW != KW || g.W != W) return false;
  const int64_t grid = (int64_t)g.N * g.G;
  if (grid > kMaxGrid) return false;
  static std::atomic<int> lds_ok{0};  // more than the default 64 KiB of dynamic LDS
  if (!lds_ok.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gconv_band_kernel<C, KH, KW, W, ROWS, MINW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Gm::LDS_BYTES) != hipSuccess) {
      *st = TC_ERR_LAUNCH;
      return true;
    }
    lds_ok.store(1, std::memory_order_release);
  }
  GconvBandArgs a{};
  a.I = g.I; a.W1 = g.W1; a.bias = g.bias; a.O = g.O;
  a.G = g.G; a.H = g.H;
  gconv_band_kernel<C, KH, KW, W, ROWS, MINW><<<dim3((unsigned)grid), dim3(WG_THREADS), Gm::LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

// ---- grouped convolution on the int8 matrix core (sliced fixed-point operands, exact int32 sums) ----
template <int W, int ROWS, int MIND>
bool try_gconv_i8(const GconvArgs& g, int force13, hipStream_t s, tc_status* st) {
  using Gm = GconvI8Geom<W, ROWS>;
  if (g.C != Gm::C || g.F != Gm::F || g.KH != Gm::KH || g.KW != Gm::KW || g.W != W) return false;
  if ((int64_t)g.H * W >= (1 << 24)) return false;  // 32-bit byte offsets inside one (image, group) block of 16 planes
  if ((g.H & 1) || (g.H - (Gm::KH - 1)) % ROWS != 0) return false;  // whole, 16-byte aligned bands only
  const int64_t bands = (int64_t)g.N * g.G * ((g.H - (Gm::KH - 1)) / ROWS);
  if (bands >= (1ll << 31)) return false;
  const int64_t grid = std::min<int64_t>(bands, 2 * (int64_t)device_cus());  // persistent: two workgroups per compute unit
  if (bands * (grid + 1) >= (1ll << 31)) return false;  // the kernel splits the bands in 32-bit arithmetic
  static std::atomic<int> lds_ok{0};  // more than the default 64 KiB of dynamic LDS
  if (!lds_ok.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gconv_i8_kernel<W, ROWS, MIND>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Gm::LDS_BYTES) != hipSuccess) {
      *st = TC_ERR_LAUNCH;
      return true;
    }
    lds_ok.store(1, std::memory_order_release);
  }
  GconvI8Args a{};
  a.I = g.I; a.W1 = g.W1; a.bias = g.bias; a.O = g.O;
  a.G = g.G; a.H = g.H; a.N = g.N;
  // Workgroups w and w + grid/2 share a compute unit; the one dispatched first wins the issue slots and runs about
  // a quarter faster, so it takes 3/5 of the pair's bands (measured at configuration 4: 121 us with an even split,
  // 117.5 us at 17/28, 118.5 at 4/7, 119.5 at 9/14).
  a.halves = (grid == 2 * (int64_t)device_cus()) ? (int)(grid / 2) : 0;
  a.num = 3;
  a.den = 5;
  a.force13 = force13;
  gconv_i8_kernel<W, ROWS, MIND><<<dim3((unsigned)grid), dim3(WG_THREADS), Gm::LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

// ---- transposed batched matmul on small per-batch matrices: flat coalesced strips through per-wavefront LDS ----
struct TbmmLdsPlan {
  int tn, tm, nx, ny, store, ks;  // what a job is and what it needs: load instructions per strip, store mode, k steps
};

// The instantiations that exist; a shape takes the first one that covers its plan.  (KS = 0: any reduction length.)
#define TC355_TBMM_LDS_VARIANTS(V) \
  V(2, 5, 3, 8, TBMM_STORE_FLAT, 7)   /* the benchmark's 26 x 72 x 26, a whole batch element per job */ \
  V(2, 5, 3, 8, TBMM_STORE_FLAT, 0)   \
  V(2, 5, 8, 16, TBMM_STORE_FLAT, 0)  \
  V(2, 1, 3, 2, TBMM_STORE_PIECES, 7) /* the same shape, one 16-column tile per job: few batch elements */ \
  V(2, 1, 3, 2, TBMM_STORE_PIECES, 0) \
  V(2, 1, 3, 2, TBMM_STORE_SCALAR, 0) \
  V(2, 2, 8, 8, TBMM_STORE_PIECES, 0) \
  V(2, 2, 8, 8, TBMM_STORE_SCALAR, 0) /* the paper's own naming of tbmm: output 26 x 26, reduction 72 */ \
  V(2, 1, 8, 8, TBMM_STORE_PIECES, 0) \
  V(2, 1, 8, 8, TBMM_STORE_SCALAR, 0) \
  V(1, 1, 4, 4, TBMM_STORE_PIECES, 0) \
  V(1, 1, 4, 4, TBMM_STORE_SCALAR, 0)

bool launch_tbmm_lds(const TbmmLdsPlan& pl, const TbmmLdsArgs& a, int64_t wgs, size_t lds, hipStream_t s, tc_status* st) {
#define TC355_TBMM_LDS_TRY(TN_, TM_, NX_, NY_, ST_, KS_)                                                       \
  if (pl.tn == TN_ && pl.tm == TM_ && pl.nx <= NX_ && pl.ny <= NY_ && pl.store == ST_ && (KS_ == 0 || pl.ks == KS_)) { \
    tbmm_lds_kernel<TN_, TM_, NX_, NY_, 1, ST_, KS_><<<dim3((unsigned)wgs), dim3(WG_THREADS), lds, s>>>(a);     \
    *st = launch_status();                                                                                     \
    return true;                                                                                               \
  }
  TC355_TBMM_LDS_VARIANTS(TC355_TBMM_LDS_TRY)
#undef TC355_TBMM_LDS_TRY
  return false;
}

// Returns false if the shape is not one for this kernel (the caller then takes the shape-generic kernels).
bool try_tbmm_lds(const float* X, const float* Y, float* Z, int64_t B, int64_t N, int64_t M, int64_t K, hipStream_t s,
                  tc_status* st) {
  if ((N * K) % 4 != 0 || (M * K) % 4 != 0 || K > 256) return false;  // strips must start and end on 16-byte boundaries
  const int cus = device_cus();
  if (cus <= 0) return false;
  const int64_t tiles_n = ceil_div(N, 16), tiles_m = ceil_div(M, 16);
  TbmmLdsPlan pl{};
  pl.tn = tiles_n >= 2 ? 2 : 1;
  const int64_t strips_n = ceil_div(tiles_n, pl.tn);
  // A whole row of tiles per job (most reuse of the X strip, contiguous results) when that still leaves two
  // wavefronts for every SIMD of the chip; with few jobs, fewer tiles per job: a shorter chain from launch to the
  // last store.
  pl.tm = 1;
  for (int c : {5, 2}) {
    if ((c == 5 ? tiles_m <= 5 && M % 4 == 0 : c <= tiles_m) && B * strips_n * ceil_div(tiles_m, c) >= 8 * (int64_t)cus) {
      pl.tm = c;
      break;
    }
  }
  const int64_t strips_m = ceil_div(tiles_m, pl.tm);
  const int64_t xrows = std::min<int64_t>(16 * pl.tn, N), yrows = std::min<int64_t>(16 * pl.tm, M);
  const int64_t xu = xrows * K / 4, yu = yrows * K / 4;  // 16-byte pieces per strip
  pl.nx = (int)ceil_div(xu, WAVE);
  pl.ny = (int)ceil_div(yu, WAVE);
  pl.store = (pl.tm == 5) ? TBMM_STORE_FLAT : (M % 4 == 0 ? TBMM_STORE_PIECES : TBMM_STORE_SCALAR);
  pl.ks = (int)ceil_div(K, 4);
  // LDS per wavefront: both strips (one spare piece: the last step of a ragged reduction reads past its row); in
  // the flat store mode the same region then holds the job's block of Z
  size_t wave_units = (size_t)(xu + yu) + 1;
  if (pl.store == TBMM_STORE_FLAT) wave_units = std::max<size_t>(wave_units, (size_t)(xrows * M / 4));
  const size_t lds = WAVES_PER_WG * wave_units * 16;
  if (lds > 64 * 1024) return false;
  if (B >= kMaxElems / (strips_n * strips_m)) return false;  // 32-bit job numbers
  TbmmLdsArgs a{};
  a.X = X; a.Y = Y; a.Z = Z;
  a.N = (int)N; a.M = (int)M; a.K = (int)K;
  a.strips_n = (int)strips_n; a.strips_m = (int)strips_m;
  a.jobs = (int)(B * strips_n * strips_m);
  a.wave_lds_units = (int)wave_units;
  // persistent wavefronts, two workgroups per compute unit (the kernel is compiled for two wavefronts per SIMD);
  // small jobs take fewer registers and less LDS, so more of their workgroups are resident at once
  const int64_t per_cu = pl.tm == 5 ? 2 : std::max<int64_t>(2, std::min<int64_t>(4, (160 * 1024) / (int64_t)lds));
  const int64_t wgs = std::min<int64_t>(ceil_div((int64_t)a.jobs, WAVES_PER_WG), per_cu * cus);
  return launch_tbmm_lds(pl, a, wgs, lds, s, st);
}

// ---- the same arithmetic for small images with 32 channels per group ----
template <int H, int W, int MIND>
bool try_gconv_i8_c32(const GconvArgs& g, hipStream_t s, tc_status* st) {
  using Gm = GconvI8C32Geom<H, W>;
  if (g.C != Gm::C || g.F != Gm::F || g.KH != Gm::KH || g.KW != Gm::KW || g.W != W || g.H != H) return false;
  if (g.N % WAVES_PER_WG != 0) return false;  // four images of a group per workgroup
  const int64_t iters = (int64_t)g.G * (g.N / WAVES_PER_WG);
  const int64_t grid = std::min<int64_t>(iters, 2 * (int64_t)device_cus());
  if (iters * (grid + 1) >= (1ll << 32)) return false;  // the kernel splits the iterations in 32-bit arithmetic
  static std::atomic<int> lds_ok{0};  // more than the default 64 KiB of dynamic LDS
  if (!lds_ok.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gconv_i8_c32_kernel<H, W, MIND>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Gm::LDS_BYTES) != hipSuccess) {
      *st = TC_ERR_LAUNCH;
      return true;
    }
    lds_ok.store(1, std::memory_order_release);
  }
  GconvI8C32Args a{};
  a.I = g.I; a.W1 = g.W1; a.bias = g.bias; a.O = g.O;
  a.G = g.G; a.N = g.N;
  gconv_i8_c32_kernel<H, W, MIND><<<dim3((unsigned)grid), dim3(WG_THREADS), Gm::LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

// ---- the same arithmetic for small images (one whole image per wavefront) ----
template <int H, int W, int MIND>
bool try_gconv_i8_small(const GconvArgs& g, hipStream_t s, tc_status* st) {
  using Gm = GconvI8SmallGeom<H, W>;
  if (g.C != Gm::C || g.F != Gm::F || g.KH != Gm::KH || g.KW != Gm::KW || g.W != W || g.H != H) return false;
  if (g.N % WAVES_PER_WG != 0) return false;  // four images of a group per workgroup
  const int64_t iters = (int64_t)g.G * (g.N / WAVES_PER_WG);
  const int64_t grid = std::min<int64_t>(iters, 2 * (int64_t)device_cus());
  if (iters * (grid + 1) >= (1ll << 32)) return false;  // the kernel splits the iterations in 32-bit arithmetic
  static std::atomic<int> lds_ok{0};  // more than the default 64 KiB of dynamic LDS
  if (!lds_ok.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gconv_i8_small_kernel<H, W, MIND>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, Gm::LDS_BYTES) != hipSuccess) {
      *st = TC_ERR_LAUNCH;
      return true;
    }
    lds_ok.store(1, std::memory_order_release);
  }
  GconvI8SmallArgs a{};
  a.I = g.I; a.W1 = g.W1; a.bias = g.bias; a.O = g.O;
  a.G = g.G; a.N = g.N;
  gconv_i8_small_kernel<H, W, MIND><<<dim3((unsigned)grid), dim3(WG_THREADS), Gm::LDS_BYTES, s>>>(a);
  *st = launch_status();
  return true;
}

}  // namespace

extern "C" {

const char* tc_status_string(tc_status s) {
  switch (s) {
    case TC_OK: return "TC_OK";
    case TC_ERR_NULL: return "TC_ERR_NULL: a required pointer is NULL";
    case TC_ERR_SHAPE: return "TC_ERR_SHAPE: an extent or an inferred extent is <= 0";
    case TC_ERR_ALIAS: return "TC_ERR_ALIAS: an output aliases an input";
    case TC_ERR_ALIGN: return "TC_ERR_ALIGN: a base pointer is not 16-byte aligned";
    case TC_ERR_WORKSPACE: return "TC_ERR_WORKSPACE: workspace missing, misaligned or too small";
    case TC_ERR_LAUNCH: return "TC_ERR_LAUNCH: the HIP runtime refused the launch";
    case TC_ERR_UNSUPPORTED: return "TC_ERR_UNSUPPORTED: extents exceed the kernels' index range";
    case TC_ERR_SCRATCH_LIMIT: return "TC_ERR_SCRATCH_LIMIT: the call needs more than the library's static scratch array holds";
  }
  return "unknown tc_status";
}

int tc355_version(void) { return 200; }

tc_status tc355_set_option(tc_option key, int64_t value) {
  switch (key) {
    case TC_OPT_INT8:
      if (value < TC_INT8_AUTO || value > TC_INT8_THIRTEEN) return TC_ERR_SHAPE;
      t_opt.int8 = value;
      return TC_OK;
    case TC_OPT_MLP_KERNEL:
      if (value < TC_MLP_AUTO || value > TC_MLP_PER_LAYER) return TC_ERR_SHAPE;
      t_opt.mlp_kernel = value;
      return TC_OK;
    case TC_OPT_MLP_SPIN_LIMIT:
      if (value < 0) return TC_ERR_SHAPE;
      t_opt.mlp_spin_limit = value;
      return TC_OK;
  }
  return TC_ERR_SHAPE;
}

int64_t tc355_get_option(tc_option key) {
  switch (key) {
    case TC_OPT_INT8: return t_opt.int8;
    case TC_OPT_MLP_KERNEL: return t_opt.mlp_kernel;
    case TC_OPT_MLP_SPIN_LIMIT: return t_opt.mlp_spin_limit;
  }
  return -1;
}

const char* tc355_last_path(void) { return t_path; }

}  // extern "C"

namespace {

// Does (B, N, M, K) belong to the shape class of the int8 transposed-matmul kernel (blocks of 128 rows of X against
// many rows of Y, long reduction)?
bool tbmm_i8_shape(int64_t B, int64_t N, int64_t M, int64_t K) {
  return N % GI8_TN == 0 && K % 4 == 0 && K >= 2 * GI8_KB && M % GI8_TM == 0 && B <= 65535 && N / GI8_TN <= 65535 &&
         (M / GI8_TM) * (N / GI8_TN) * B >= 128;
}

// Does slicing X once, in a kernel of its own, pay?  The extra launch costs 2-3 us; what it saves grows with the number
// of workgroups that would each slice X (M / 64) and with the length of the reduction.  Measured: 138 -> 128 us at
// (B,N,M,K) = (1,128,16384,4096), 19.8 -> 22.3 us at (2,256,4096,512).
bool tbmm_presliced_pays(int64_t B, int64_t N, int64_t M, int64_t K) {
  return M / GI8_TM >= 128 && K / GI8_KB >= 16 && B * (N / GI8_TN) <= 65535 && ceil_div(K, GI8_KB) <= kMaxGrid;
}

// bytes of X sliced once for the int8 kernel: digit records, then inverse scales
size_t tbmm_ws_bytes(int64_t B, int64_t N, int64_t K) {
  const int64_t blocks = B * (N / GI8_TN) * ceil_div(K, GI8_KB);
  return (size_t)(blocks * (GI8_XD_BYTES + GI8_XINV_BYTES));
}

tc_status tbmm_run(const float* X, const float* Y, float* Z, int64_t B, int64_t N, int64_t M, int64_t K, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  if (!X || !Y || !Z) return TC_ERR_NULL;
  if (B < 0 || N <= 0 || M <= 0 || K <= 0) return TC_ERR_SHAPE;
  if (Z == X || Z == Y) return TC_ERR_ALIAS;
  if (misaligned(X) || misaligned(Y) || misaligned(Z)) return TC_ERR_ALIGN;
  if (B >= kMaxElems || prod_reaches({N, K}, kMaxElems) || prod_reaches({M, K}, kMaxElems) || prod_reaches({N, M}, kMaxElems))
    return TC_ERR_UNSUPPORTED;
  if (B == 0) return TC_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  // The paper's largest tmm shape class (blocks of 128 rows against many, long reduction) on the int8 matrix core;
  // option TC_INT8_OFF keeps it on the fp64 kernels.
  if (tbmm_i8_shape(B, N, M, K) && t_opt.int8 != TC_INT8_OFF) {
    static std::atomic<int> lds_ok{0};  // more than the default 64 KiB of dynamic LDS
    if (!lds_ok.load(std::memory_order_acquire)) {
      const void* kernels[4] = {reinterpret_cast<const void*>(gemm_i8_kernel<2, false>), reinterpret_cast<const void*>(gemm_i8_kernel<3, false>),
                                reinterpret_cast<const void*>(gemm_i8_kernel<2, true>), reinterpret_cast<const void*>(gemm_i8_kernel<3, true>)};
      for (const void* k : kernels)
        if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, GI8_LDS_BYTES) != hipSuccess) return TC_ERR_LAUNCH;
      lds_ok.store(1, std::memory_order_release);
    }
    GemmI8Args g{};
    g.X = X; g.Y = Y; g.Z = Z; g.M = (int)M; g.K = (int)K;
    const dim3 grid((unsigned)(M / GI8_TM), (unsigned)B, (unsigned)(N / GI8_TN));
    const bool ten = t_opt.int8 == TC_INT8_TEN;  // 13 digit products unless the caller has said that 10 will do
    // With a workspace X is sliced once, by a kernel of its own, instead of by every workgroup that reads it.
    if (workspace && tbmm_presliced_pays(B, N, M, K) && workspace_bytes >= tbmm_ws_bytes(B, N, K)) {
      const int64_t rblocks = B * (N / GI8_TN), nb = ceil_div(K, GI8_KB);
      i4* xd = static_cast<i4*>(workspace);
      double* xinv = reinterpret_cast<double*>(static_cast<char*>(workspace) + rblocks * nb * GI8_XD_BYTES);
      gemm_i8_slice_x_kernel<<<dim3((unsigned)nb, (unsigned)rblocks), dim3(GI8_THREADS), 0, s>>>(X, (int)K, xd, xinv);
      const tc_status st = launch_status();
      if (st != TC_OK) return st;
      g.Xd = xd; g.Xinv = xinv;
      if (ten) gemm_i8_kernel<3, true><<<grid, dim3(GI8_THREADS), GI8_LDS_BYTES, s>>>(g);
      else gemm_i8_kernel<2, true><<<grid, dim3(GI8_THREADS), GI8_LDS_BYTES, s>>>(g);
      return took("tbmm:i8_presliced", launch_status());
    }
    if (ten) gemm_i8_kernel<3, false><<<grid, dim3(GI8_THREADS), GI8_LDS_BYTES, s>>>(g);
    else gemm_i8_kernel<2, false><<<grid, dim3(GI8_THREADS), GI8_LDS_BYTES, s>>>(g);
    return took("tbmm:i8", launch_status());
  }

  {
    tc_status st = TC_OK;
    if (try_tbmm_lds(X, Y, Z, B, N, M, K, s, &st)) return took("tbmm:lds", st);
  }

  GemmArgs a{};
  a.A = X; a.Bm = Y; a.bias = nullptr; a.C = Z; a.C64 = nullptr;
  a.strideA = N * K; a.strideB = M * K; a.strideC = N * M;
  a.N = (int)N; a.M = (int)M; a.K = (int)K;
  const int tm = pick_strip(M, B * ceil_div(N, 16) * ceil_div(M, 16));
  return launch_gemm<float, EPI_NONE>(a, B, tm, s);  // records tbmm:tile, tbmm:splitk or tbmm:wave
}

}  // namespace

extern "C" {

tc_status tc_tbmm(const float* X, const float* Y, float* Z, int64_t B, int64_t N, int64_t M, int64_t K,
                  void* hip_stream) {
  return tbmm_run(X, Y, Z, B, N, M, K, nullptr, 0, hip_stream);
}

size_t tc_tbmm_workspace_bytes(int64_t B, int64_t N, int64_t M, int64_t K) {
  if (B <= 0 || N <= 0 || M <= 0 || K <= 0 || B >= kMaxElems || prod_reaches({N, K}, kMaxElems)) return 0;
  if (!tbmm_i8_shape(B, N, M, K) || !tbmm_presliced_pays(B, N, M, K)) return 0;
  return tbmm_ws_bytes(B, N, K);
}

tc_status tc_tbmm_ws(const float* X, const float* Y, float* Z, int64_t B, int64_t N, int64_t M, int64_t K,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (workspace && misaligned(workspace)) return TC_ERR_ALIGN;
  if (workspace && (workspace == X || workspace == Y || workspace == Z)) return TC_ERR_ALIAS;
  return tbmm_run(X, Y, Z, B, N, M, K, workspace, workspace_bytes, hip_stream);
}

size_t tc_mlp_fcrelu_workspace_bytes(int64_t batch, int32_t n_layers, const int64_t* dims) {
  if (!dims || batch < 0 || n_layers <= 0 || n_layers > MLP_MAX_LAYERS) return 0;
  if (n_layers == 1) return 0;
  size_t total = mlp_sync_bytes();  // synchronisation words first
  for (int l = 0; l + 1 < n_layers; l++) {
    if (dims[l + 1] <= 0) return 0;
    total += mlp_act_bytes(batch, dims[l + 1]);
  }
  return total;
}

}  // extern "C"

namespace {

// Scratch of tc_mlp_fcrelu_static: one array per GPU that the library runs on, held until the process ends.
// In host code the array's name is only a stand-in; its device address comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[TC_MLP_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current device (looked up once per device), or nullptr on failure.
void* static_scratch_ptr() {
  static std::atomic<void*> cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  void* ptr = cache[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    cache[dev].store(ptr, std::memory_order_release);
  }
  return ptr;
}

// Both MLP entry points: validation, then the fused kernel or one launch per layer.  `workspace` is device memory.
tc_status mlp_run(const float* I, int64_t batch, int32_t n_layers, const int64_t* dims, const float* const* W,
                  const float* const* bias, float* const* O, void* workspace, size_t workspace_bytes,
                  bool static_scratch, void* hip_stream) {
  if (!I || !dims || !W || !bias || !O) return TC_ERR_NULL;
  if (batch < 0 || n_layers <= 0 || n_layers > MLP_MAX_LAYERS) return TC_ERR_SHAPE;
  for (int l = 0; l <= n_layers; l++)
    if (dims[l] <= 0) return TC_ERR_SHAPE;
  for (int l = 0; l < n_layers; l++)
    if (!W[l] || !bias[l]) return TC_ERR_NULL;
  if (!O[n_layers - 1]) return TC_ERR_NULL;
  if (misaligned(I)) return TC_ERR_ALIGN;
  for (int l = 0; l < n_layers; l++) {
    if (misaligned(W[l]) || misaligned(bias[l]) || (O[l] && misaligned(O[l]))) return TC_ERR_ALIGN;
    if (O[l] && (O[l] == I)) return TC_ERR_ALIAS;
    for (int m = 0; m < n_layers; m++) {
      if (O[l] && (O[l] == W[m] || O[l] == bias[m])) return TC_ERR_ALIAS;
      if (O[l] && m != l && O[l] == O[m]) return TC_ERR_ALIAS;
    }
    if (prod_reaches({dims[l], dims[l + 1]}, kMaxElems) || prod_reaches({std::max<int64_t>(batch, 1), dims[l]}, kMaxElems) ||
        prod_reaches({std::max<int64_t>(batch, 1), dims[l + 1]}, kMaxElems))
      return TC_ERR_UNSUPPORTED;
  }
  const size_t need = tc_mlp_fcrelu_workspace_bytes(batch, n_layers, dims);
  if (static_scratch) {
    if (need > TC_MLP_STATIC_SCRATCH_BYTES) return TC_ERR_SCRATCH_LIMIT;
    if (batch == 0) return TC_OK;
    if (need > 0) {
      workspace = static_scratch_ptr();
      workspace_bytes = TC_MLP_STATIC_SCRATCH_BYTES;
      if (!workspace) return TC_ERR_LAUNCH;
    }
  }
  if (need > 0 && (!workspace || misaligned(workspace, 256) || workspace_bytes < need)) return TC_ERR_WORKSPACE;
  if (batch == 0) return TC_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  // workspace: [synchronisation words | fp64 activations of layer 0 | layer 1 | ...]
  char* ws = static_cast<char*>(workspace);
  double* act[MLP_MAX_LAYERS] = {};
  {
    char* pws = ws + mlp_sync_bytes();
    for (int l = 0; l + 1 < n_layers; l++) {
      act[l] = reinterpret_cast<double*>(pws);
      pws += mlp_act_bytes(batch, dims[l + 1]);
    }
  }

  // One persistent kernel for the whole chain when every reduction extent allows 16-byte loads.
  bool fused = t_opt.mlp_kernel != TC_MLP_PER_LAYER;
  for (int l = 0; l < n_layers; l++) fused = fused && (dims[l] % 4 == 0);
  // the fused kernel addresses its operands (fp64 activations, fp32 weights) with 32-bit byte offsets
  for (int l = 0; l < n_layers; l++)
    fused = fused && batch * dims[l] * 8 < (1ll << 32) && dims[l + 1] * dims[l] * 4 < (1ll << 32);
  // Large batches: when every layer fills the chip with 64 x 64 blocks, one LDS-tiled launch per layer (70 % of the
  // fp64 matrix peak) beats the fused kernel's 16 x 16 tiles (43 %), and the launches no longer matter.
  if (n_layers > 1 && t_opt.mlp_kernel == TC_MLP_AUTO) {
    int64_t min_blocks = INT64_MAX;
    for (int l = 0; l < n_layers; l++) min_blocks = std::min(min_blocks, ceil_div(batch, GT_BM) * ceil_div(dims[l + 1], GT_BN));
    if (min_blocks >= 256) fused = false;
  }
  const int cus = device_cus();
  // Small batches with reductions of at most 1024: one workgroup per compute unit, every XCD's workgroups own an eighth
  // of the column tiles of every layer (mlp_rows.hpp).  Option TC_OPT_MLP_KERNEL = TC_MLP_TILES keeps the tile-stream
  // kernel below.
  if (fused && cus >= MR_SHARES) {
    const int64_t G = ceil_div(batch, 16);
    const int64_t nwg = std::min<int64_t>(cus, MR_MAX_WG) / MR_SHARES * MR_SHARES;
    int64_t max_ct = 1;  // most column tiles of any layer whose output is handed on
    for (int l = 0; l + 1 < n_layers; l++) max_ct = std::max(max_ct, ceil_div(dims[l + 1], 16));
    const int64_t fstride = 4 * max_ct;
    bool rows = t_opt.mlp_kernel != TC_MLP_TILES && G <= 64 &&
                (int64_t)(n_layers - 1) * G * fstride <= (int64_t)(MLP_MAX_LAYERS - 1) * MLP_BAR_WORDS;
    for (int l = 0; l < n_layers && rows; l++)
      rows = (dims[l] == 128 || dims[l] == 256 || dims[l] == 512 || dims[l] == 1024) &&
             mr_deal((int)ceil_div(dims[l + 1], 16), (int)G, (int)(nwg / MR_SHARES)).fits;
    if (rows) {
      MlpRowsArgs a{};
      a.I = I;
      for (int l = 0; l < n_layers; l++) {
        a.W[l] = W[l]; a.bias[l] = bias[l]; a.O[l] = O[l]; a.act[l] = act[l];
      }
      for (int l = 0; l <= n_layers; l++) a.dims[l] = (int)dims[l];
      a.batch = (int)batch; a.n_layers = n_layers; a.groups = (int)G; a.fstride = (int)fstride;
      a.sync = reinterpret_cast<unsigned*>(ws);
      a.token = next_token();
      a.spin_limit = (unsigned)std::max<int64_t>(0, std::min<int64_t>(t_opt.mlp_spin_limit, 0xffffffffll));
      static std::atomic<int> lds_ok{0};  // more than the default 64 KiB of dynamic LDS
      if (!lds_ok.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_rows_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                MR_LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_rows_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                MR_LDS_BYTES) != hipSuccess)
          return TC_ERR_LAUNCH;
        lds_ok.store(1, std::memory_order_release);
      }
      bool wide = true;  // every reduction extent 512 or 1024: the kernel that carries only those layer bodies
      for (int l = 0; l < n_layers; l++) wide = wide && dims[l] >= 512;
      if (wide) mlp_rows_kernel<true><<<dim3((unsigned)nwg), dim3(MR_THREADS), MR_LDS_BYTES, s>>>(a);
      else mlp_rows_kernel<false><<<dim3((unsigned)nwg), dim3(MR_THREADS), MR_LDS_BYTES, s>>>(a);
      return took("mlp:rows", launch_status());
    }
  }
  if (fused && cus > 0) {
    MlpArgs a{};
    a.I = I;
    int64_t max_jobs = 1;
    for (int l = 0; l < n_layers; l++) {
      a.W[l] = W[l]; a.bias[l] = bias[l]; a.O[l] = O[l]; a.act[l] = act[l];
      max_jobs = std::max<int64_t>(max_jobs, ceil_div(batch, 16) * ceil_div(dims[l + 1], 16));
    }
    for (int l = 0; l <= n_layers; l++) a.dims[l] = (int)dims[l];
    a.batch = (int)batch; a.n_layers = n_layers;
    a.sync = reinterpret_cast<unsigned*>(ws);
    a.token = next_token();
    a.spin_limit = (unsigned)std::max<int64_t>(1, std::min<int64_t>(t_opt.mlp_spin_limit, 0xffffffffll));
    const unsigned nwg = (unsigned)std::min<int64_t>(std::min(2 * cus, MLP_FANIN * MLP_GROUPS), max_jobs);  // teams of four wavefronts, all resident: two per compute unit
    static std::atomic<int> lds_ok{0};  // the kernel stages more than the default 64 KiB of LDS
    if (!lds_ok.load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_fused_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, MLP_TEAMS * MLP_LDS_BYTES) != hipSuccess)
        return TC_ERR_LAUNCH;
      lds_ok.store(1, std::memory_order_release);
    }
    // nwg teams of four wavefronts; MLP_TEAMS of them share a workgroup
    mlp_fused_kernel<<<dim3((nwg + MLP_TEAMS - 1) / MLP_TEAMS), dim3(MLP_TEAMS * WG_THREADS), MLP_TEAMS * MLP_LDS_BYTES, s>>>(a);
    return took("mlp:tiles", launch_status());
  }

  // Otherwise one launch per layer through the shape-generic contraction.
  const void* in = I;
  for (int l = 0; l < n_layers; l++) {
    GemmArgs a{};
    a.A = in; a.Bm = W[l]; a.bias = bias[l]; a.C = O[l]; a.C64 = act[l];
    a.strideA = 0; a.strideB = 0; a.strideC = 0;
    a.N = (int)batch; a.M = (int)dims[l + 1]; a.K = (int)dims[l];
    const int tm = pick_strip(dims[l + 1], ceil_div(batch, 16) * ceil_div(dims[l + 1], 16));
    const tc_status st = (l == 0) ? launch_gemm<float, EPI_BIAS_RELU>(a, 1, tm, s)
                                  : launch_gemm<double, EPI_BIAS_RELU>(a, 1, tm, s);
    if (st != TC_OK) return st;
    in = act[l];
  }
  return took("mlp:per_layer", TC_OK);
}

// Strided convolution on the fp64 matrix core (sconv_tile.hpp): blocks of 64 filters x 64 or 32 pixels.
tc_status launch_sconv_tile(SconvArgs a, hipStream_t s) {
  a.tiles_f = (int)ceil_div(a.F, SC_BF);
  // 64-pixel blocks when there are at least two of them per compute unit, else 32-pixel blocks (twice as many)
  const bool wide = (int64_t)a.tiles_f * ceil_div(a.P, 64) >= 2 * (int64_t)std::max(1, device_cus());
  const int64_t grid = (int64_t)a.tiles_f * ceil_div(a.P, wide ? 64 : 32);
  if (grid > kMaxGrid) return TC_ERR_UNSUPPORTED;
  const dim3 gd((unsigned)grid), bd(WG_THREADS);
  if (wide) {
    if (a.K % 4 == 0) sconv_tile_kernel<4, 64><<<gd, bd, SconvGeom<64>::LDS_BYTES, s>>>(a);
    else sconv_tile_kernel<1, 64><<<gd, bd, SconvGeom<64>::LDS_BYTES, s>>>(a);
  } else {
    if (a.K % 4 == 0) sconv_tile_kernel<4, 32><<<gd, bd, SconvGeom<32>::LDS_BYTES, s>>>(a);
    else sconv_tile_kernel<1, 32><<<gd, bd, SconvGeom<32>::LDS_BYTES, s>>>(a);
  }
  return launch_status();
}

// Strided convolution on the int8 matrix core (sconv_i8.hpp): TF filters against 16 * NT pixels per workgroup.
template <int TF, int NT>
tc_status launch_sconv_i8(const SconvI8Args& a, int64_t blocks, dim3 grid, bool ten, hipStream_t s) {
  constexpr int kLdsMax = 160 * 1024;
  static std::atomic<int> lds_ok{0};  // more than the default 64 KiB of dynamic LDS
  if (!lds_ok.load(std::memory_order_acquire)) {
    const void* kernels[2] = {reinterpret_cast<const void*>(sconv_i8_kernel<TF, NT, 2>),
                              reinterpret_cast<const void*>(sconv_i8_kernel<TF, NT, 3>)};
    for (const void* k : kernels)
      if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMax) != hipSuccess) return TC_ERR_LAUNCH;
    lds_ok.store(1, std::memory_order_release);
  }
  const size_t lds = (size_t)SconvI8Geom<TF, NT>::lds_bytes(blocks);
  if (lds > (size_t)kLdsMax) return TC_ERR_LAUNCH;  // (the caller has checked)
  if (ten) sconv_i8_kernel<TF, NT, 3><<<grid, dim3(SI8_THREADS), lds, s>>>(a);
  else sconv_i8_kernel<TF, NT, 2><<<grid, dim3(SI8_THREADS), lds, s>>>(a);
  return launch_status();
}

// LDS bytes of the kernel for tf filters and nt pixel tiles per workgroup (the geometry depends on tf + 16 nt only)
int64_t sconv_i8_lds_bytes(int tf, int nt, int64_t blocks) {
  const int64_t rows = tf + 16 * nt;
  return 4 * rows * SI8_RS + rows * 8 + 2 * 16 * nt * 4 + blocks * SI8_KB * 4;
}

// Takes the call if the shape is one the int8 kernel is built for: a multiple of 32 filters, a reduction C * KH * KW
// that is a multiple of 4 and at least 256 taps (two blocks), operands that 32-bit offsets reach, a table of tap
// offsets that fits LDS beside the digit planes (about 17,000 taps).  Measured faster than the fp64 kernel from a
// single 8 x 8 image up.
bool try_sconv_i8(const SconvI8Args& a, int64_t N, hipStream_t s, tc_status* st) {  // a.G groups of a.C channels and a.F filters
  if (t_opt.int8 == TC_INT8_OFF) return false;
  if (a.F % 32 != 0 || a.K % 4 != 0 || a.K < 256) return false;
  if (prod_reaches({N, a.G, a.C, a.H, a.W}, (int64_t)1 << 30)) return false;            // 32-bit byte offsets into I
  if (prod_reaches({N, a.G, a.F, a.OH, a.OW}, (int64_t)1 << 31)) return false;          // 32-bit element offsets into O
  if (a.G > 65535) return false;
  // 128 filters per workgroup and 1 .. 4 pixel tiles, or (a multiple of 64 filters only) 64 filters and 2, 4, 6, 8,
  // or (a multiple of 32 only) 32 filters and 4, 8, 12
  const int tf = a.F % 128 == 0 ? 128 : (a.F % 64 == 0 ? 64 : 32), nt_step = 128 / tf, nt_max = tf == 32 ? 12 : 4 * nt_step;
  const int64_t blocks = ceil_div(a.K, SI8_KB), units = ceil_div(a.P, 16), fblocks = a.F / tf;
  // pixel tiles per workgroup: as few rounds of workgroups as the largest tile allows, then the smallest tile
  // that still makes that number of rounds
  const int64_t per_round = std::max<int64_t>(1, device_cus() / (fblocks * a.G));
  const int64_t rounds = ceil_div(units, nt_max * per_round);
  int nt = (int)ceil_div(ceil_div(units, rounds * per_round), nt_step) * nt_step;
  nt = std::min(nt_max, std::max(nt_step, nt));
  while (nt > nt_step && sconv_i8_lds_bytes(tf, nt, blocks) > 160 * 1024) nt -= nt_step;
  if (sconv_i8_lds_bytes(tf, nt, blocks) > 160 * 1024) return false;
  const int64_t gx = ceil_div(units, nt);
  if (gx > kMaxGrid || fblocks > 65535) return false;
  const dim3 grid((unsigned)gx, (unsigned)fblocks, (unsigned)a.G);
  const bool ten = t_opt.int8 == TC_INT8_TEN;  // 13 digit products unless the caller has said that 10 will do
  if (tf == 128) {
    switch (nt) {
      case 1: *st = launch_sconv_i8<128, 1>(a, blocks, grid, ten, s); break;
      case 2: *st = launch_sconv_i8<128, 2>(a, blocks, grid, ten, s); break;
      case 3: *st = launch_sconv_i8<128, 3>(a, blocks, grid, ten, s); break;
      default: *st = launch_sconv_i8<128, 4>(a, blocks, grid, ten, s); break;
    }
  } else if (tf == 64) {
    switch (nt) {
      case 2: *st = launch_sconv_i8<64, 2>(a, blocks, grid, ten, s); break;
      case 4: *st = launch_sconv_i8<64, 4>(a, blocks, grid, ten, s); break;
      case 6: *st = launch_sconv_i8<64, 6>(a, blocks, grid, ten, s); break;
      default: *st = launch_sconv_i8<64, 8>(a, blocks, grid, ten, s); break;
    }
  } else {
    switch (nt) {
      case 4: *st = launch_sconv_i8<32, 4>(a, blocks, grid, ten, s); break;
      case 8: *st = launch_sconv_i8<32, 8>(a, blocks, grid, ten, s); break;
      default: *st = launch_sconv_i8<32, 12>(a, blocks, grid, ten, s); break;
    }
  }
  return true;
}

}  // namespace

extern "C" {

tc_status tc_mlp_fcrelu(const float* I, int64_t batch, int32_t n_layers, const int64_t* dims,
                        const float* const* W, const float* const* bias, float* const* O, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  return mlp_run(I, batch, n_layers, dims, W, bias, O, workspace, workspace_bytes, false, hip_stream);
}

tc_status tc_mlp_fcrelu_static(const float* I, int64_t batch, int32_t n_layers, const int64_t* dims,
                               const float* const* W, const float* const* bias, float* const* O,
                               void* hip_stream) {
  return mlp_run(I, batch, n_layers, dims, W, bias, O, nullptr, 0, true, hip_stream);
}

tc_status tc_group_conv_infer(int64_t H, int64_t W, int64_t KH, int64_t KW, int64_t* OH, int64_t* OW) {
  if (!OH || !OW) return TC_ERR_NULL;
  if (H <= 0 || W <= 0 || KH <= 0 || KW <= 0) return TC_ERR_SHAPE;
  if (H - KH + 1 <= 0 || W - KW + 1 <= 0) return TC_ERR_SHAPE;
  *OH = H - KH + 1;
  *OW = W - KW + 1;
  return TC_OK;
}

tc_status tc_group_conv(const float* I, const float* W1, const float* bias, float* O, int64_t N, int64_t G,
                        int64_t C, int64_t F, int64_t H, int64_t W, int64_t KH, int64_t KW, void* hip_stream) {
  if (!I || !W1 || !O) return TC_ERR_NULL;
  if (N < 0 || G <= 0 || C <= 0 || F <= 0) return TC_ERR_SHAPE;
  int64_t OH, OW;
  const tc_status inf = tc_group_conv_infer(H, W, KH, KW, &OH, &OW);
  if (inf != TC_OK) return inf;
  if (O == I || O == W1 || (bias && O == bias)) return TC_ERR_ALIAS;
  if (misaligned(I) || misaligned(W1) || misaligned(O) || (bias && misaligned(bias))) return TC_ERR_ALIGN;
  if (N >= kMaxElems || prod_reaches({C, H, W}, kMaxElems) || prod_reaches({F, OH, OW}, kMaxElems) || prod_reaches({C, KH, KW}, kMaxElems) ||
      prod_reaches({G, F, C, KH, KW}, kMaxElems) || G >= kMaxElems / 16 || F >= kMaxElems / 16)
    return TC_ERR_UNSUPPORTED;
  if (N == 0) return TC_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  GconvArgs a{};
  a.I = I; a.W1 = W1; a.bias = bias; a.O = O;
  a.N = (int)N; a.G = (int)G; a.C = (int)C; a.F = (int)F; a.H = (int)H; a.W = (int)W;
  a.KH = (int)KH; a.KW = (int)KW; a.OH = (int)OH; a.OW = (int)OW;
  tc_status st = TC_OK;
  // Option TC_OPT_INT8: AUTO = the int8 path where it applies, with the thirteenth to tenth digit products added for
  // heavy-tailed blocks; TEN / THIRTEEN = the same with 10 / 13 products throughout; OFF = the fp64 path for every shape.
  const int64_t i8 = t_opt.int8;
  const int force13 = i8 == TC_INT8_THIRTEEN ? 1 : (i8 == TC_INT8_TEN ? -1 : 0);
  if (i8 != TC_INT8_OFF) {
    if (try_gconv_i8<58, 8, 3>(a, force13, s, &st)) return took("gconv:i8", st);
    if (i8 == TC_INT8_TEN) {
      if (try_gconv_i8_small<14, 14, 3>(a, s, &st)) return took("gconv:i8_small", st);  // the paper's (32,32,16,16,14,14)
      if (try_gconv_i8_c32<7, 7, 3>(a, s, &st)) return took("gconv:i8_c32", st);     // the paper's (32,32,32,32,7,7)
      if (try_gconv_i8_small<16, 16, 3>(a, s, &st)) return took("gconv:i8_small", st);  // the first with a border of one pixel
    } else {
      if (try_gconv_i8_small<14, 14, 2>(a, s, &st)) return took("gconv:i8_small", st);
      if (try_gconv_i8_c32<7, 7, 2>(a, s, &st)) return took("gconv:i8_c32", st);
      if (try_gconv_i8_small<16, 16, 2>(a, s, &st)) return took("gconv:i8_small", st);
    }
    // groups with a multiple of 64 filters and at least 256 taps (G = 1: the plain convolution of Section 3): the
    // strided convolution's int8 kernel with stride 1, one grid plane per group
    if (C * KH * KW < kMaxElems && N * OH * OW < kMaxElems) {
      SconvI8Args e{};
      e.I = I; e.Wt = W1; e.bias = bias; e.O = O;
      e.C = (int)C; e.F = (int)F; e.H = (int)H; e.W = (int)W; e.KH = (int)KH; e.KW = (int)KW; e.sh = 1; e.sw = 1;
      e.OH = (int)OH; e.OW = (int)OW; e.K = (int)(C * KH * KW); e.P = (int)(N * OH * OW); e.G = (int)G;
      if (try_sconv_i8(e, N, s, &st)) return took("gconv:i8_taps", st);
    }
  }
  if (try_gconv_band<16, 3, 3, 58, 8, 2>(a, s, &st)) return took("gconv:band", st);
  if (try_gconv_band<16, 3, 3, 14, 12, 2>(a, s, &st)) return took("gconv:band", st);  // the paper's (32,32,16,16,14,14): the whole image is one band
  if (try_gconv_quad<4, 4, 3, 3, 56, 16, 4>(a, s, &st)) return took("gconv:quad", st);    // the paper's (32,32,4,4,56,56)
  if (try_gconv_quad<8, 8, 3, 3, 28, 26, 3>(a, s, &st)) return took("gconv:quad", st);    // the paper's (32,32,8,8,28,28): one band
  if (try_gconv_quad<4, 4, 3, 3, 58, 16, 4>(a, s, &st)) return took("gconv:quad", st);    // the same two with a border of one pixel
  if (try_gconv_quad<8, 8, 3, 3, 30, 14, 3>(a, s, &st)) return took("gconv:quad", st);
  if (try_gconv_tiny<32, 32, 3, 3, 7, 7>(a, s, &st)) return took("gconv:tiny", st);       // the paper's (32,32,32,32,7,7)
  if (try_gconv_lds<16, 16, 3, 3, 7>(a, s, &st)) return took("gconv:lds", st);
  // G = 1 is the plain convolution of Section 3: the strided convolution's fp64 kernel (implicit contraction over
  // all pixels of the batch in blocks of 64 x 64) where there are at least 64 filters and 64 taps to fill its blocks
  if (G == 1 && F >= 64 && C * KH * KW >= 64 && !prod_reaches({N, C, H, W}, kMaxElems) && !prod_reaches({N, F, OH, OW}, kMaxElems) &&
      !prod_reaches({N, OH, OW}, kMaxElems)) {
    SconvArgs e{};
    e.I = I; e.Wt = W1; e.bias = bias; e.O = O;
    e.N = (int)N; e.C = (int)C; e.F = (int)F; e.H = (int)H; e.W = (int)W; e.KH = (int)KH; e.KW = (int)KW;
    e.sh = 1; e.sw = 1; e.OH = (int)OH; e.OW = (int)OW; e.K = (int)(C * KH * KW); e.P = (int)(N * OH * OW);
    return took("gconv:tile", launch_sconv_tile(e, s));
  }
  t_path = "gconv:wave";
  // generic kernel: a wavefront takes 16 filters x a strip of 16*TP pixels; small images take a narrower strip
  const int64_t tiles_p = ceil_div(OH * OW, 16);
  const int tp = tiles_p >= 4 ? 4 : (tiles_p >= 2 ? 2 : 1);
  a.tiles_f = (int)ceil_div(F, 16);
  a.strips_p = (int)ceil_div(OH * OW, 16 * tp);
  a.jobs = N * G * a.tiles_f * a.strips_p;
  const int64_t grid = ceil_div(a.jobs, WAVES_PER_WG);
  if (grid > kMaxGrid) return TC_ERR_UNSUPPORTED;
  const dim3 gd((unsigned)grid), bd(WG_THREADS);
  if (tp == 4) gconv_wave_kernel<4><<<gd, bd, 0, s>>>(a);
  else if (tp == 2) gconv_wave_kernel<2><<<gd, bd, 0, s>>>(a);
  else gconv_wave_kernel<1><<<gd, bd, 0, s>>>(a);
  return launch_status();
}

tc_status tc_kron(const float* W1, const float* W2, const float* X, float* Y, int64_t B, int64_t I, int64_t K,
                  int64_t J, int64_t L, void* hip_stream) {
  if (!W1 || !W2 || !X || !Y) return TC_ERR_NULL;
  if (B < 0 || I <= 0 || K <= 0 || J <= 0 || L <= 0) return TC_ERR_SHAPE;
  if (Y == W1 || Y == W2 || Y == X) return TC_ERR_ALIAS;
  if (misaligned(W1) || misaligned(W2) || misaligned(X) || misaligned(Y)) return TC_ERR_ALIGN;
  if (B >= kMaxElems || prod_reaches({I, K}, kMaxElems) || prod_reaches({J, L}, kMaxElems) || prod_reaches({K, L}, kMaxElems) ||
      prod_reaches({I, J}, kMaxElems))
    return TC_ERR_UNSUPPORTED;
  if (B == 0) return TC_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  KronArgs a{};
  a.W1 = W1; a.W2 = W2; a.X = X; a.Y = Y;
  a.I = (int)I; a.K = (int)K; a.J = (int)J; a.L = (int)L;
  if (K == 64 && L == 64 && J == 64) {
    KronLdsArgs f{};
    f.W1 = W1; f.W2 = W2; f.X = X; f.Y = Y;
    f.I = (int)I;
    f.iblocks = (int)ceil_div(I, 64);
    const int64_t fgrid = B * f.iblocks;
    if (fgrid <= kMaxGrid) {
      kron_lds_kernel<64, 64, 64><<<dim3((unsigned)fgrid), dim3(WG_THREADS), 0, s>>>(f);
      return took("kron:lds", launch_status());
    }
  }
  constexpr int TJ = 4;
  a.tiles_i = (int)ceil_div(I, 16);
  a.blocks_j = (int)ceil_div(J, 16 * TJ);
  a.jobs = B * a.tiles_i * a.blocks_j;
  const int64_t grid = ceil_div(a.jobs, WAVES_PER_WG);
  if (grid > kMaxGrid) return TC_ERR_UNSUPPORTED;
  kron_wave_kernel<TJ><<<dim3((unsigned)grid), dim3(WG_THREADS), 0, s>>>(a);
  return took("kron:wave", launch_status());
}

tc_status tc_sconv2d_infer(int64_t H, int64_t W, int64_t KH, int64_t KW, int64_t sh, int64_t sw, int64_t* OH,
                           int64_t* OW) {
  if (!OH || !OW) return TC_ERR_NULL;
  if (H <= 0 || W <= 0 || KH <= 0 || KW <= 0 || sh <= 0 || sw <= 0) return TC_ERR_SHAPE;
  if (H < KH || W < KW) return TC_ERR_SHAPE;
  *OH = (H - KH) / sh + 1;
  *OW = (W - KW) / sw + 1;
  return TC_OK;
}

tc_status tc_sconv2d(const float* I, const float* Wt, const float* bias, float* O, int64_t N, int64_t C, int64_t F,
                     int64_t H, int64_t W, int64_t KH, int64_t KW, int64_t sh, int64_t sw, void* hip_stream) {
  if (!I || !Wt || !O) return TC_ERR_NULL;
  if (N < 0 || C <= 0 || F <= 0) return TC_ERR_SHAPE;
  int64_t OH, OW;
  const tc_status inf = tc_sconv2d_infer(H, W, KH, KW, sh, sw, &OH, &OW);
  if (inf != TC_OK) return inf;
  if (O == I || O == Wt || (bias && O == bias)) return TC_ERR_ALIAS;
  if (misaligned(I) || misaligned(Wt) || misaligned(O) || (bias && misaligned(bias))) return TC_ERR_ALIGN;
  const int64_t N1 = std::max<int64_t>(N, 1);
  if (prod_reaches({N1, C, H, W}, kMaxElems) || prod_reaches({F, C, KH, KW}, kMaxElems) ||
      prod_reaches({N1, OH, OW}, kMaxElems) || prod_reaches({F, OH, OW}, kMaxElems) || sh >= kMaxElems || sw >= kMaxElems)
    return TC_ERR_UNSUPPORTED;
  const int64_t K = C * KH * KW;
  if (N == 0) return TC_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  {
    SconvI8Args e{};
    e.I = I; e.Wt = Wt; e.bias = bias; e.O = O;
    e.C = (int)C; e.F = (int)F; e.H = (int)H; e.W = (int)W; e.KH = (int)KH; e.KW = (int)KW; e.sh = (int)sh; e.sw = (int)sw;
    e.OH = (int)OH; e.OW = (int)OW;
    e.K = (int)K; e.P = (int)(N * OH * OW); e.G = 1;
    tc_status st = TC_OK;
    if (try_sconv_i8(e, N, s, &st)) return took("sconv:i8", st);
  }

  SconvArgs a{};
  a.I = I; a.Wt = Wt; a.bias = bias; a.O = O;
  a.N = (int)N; a.C = (int)C; a.F = (int)F; a.H = (int)H; a.W = (int)W; a.KH = (int)KH; a.KW = (int)KW;
  a.sh = (int)sh; a.sw = (int)sw; a.OH = (int)OH; a.OW = (int)OW;
  a.K = (int)K; a.P = (int)(N * OH * OW);
  return took("sconv:tile", launch_sconv_tile(a, s));
}

tc_status tc_lut(int32_t n_tables, const float* const* LUT, const int32_t* const* Idx, float* const* O,
                 const int64_t* E, const int64_t* L, int64_t D, int64_t B, void* hip_stream) {
  if (!LUT || !Idx || !O || !E || !L) return TC_ERR_NULL;
  if (n_tables <= 0 || n_tables > LUT_MAX_TABLES || D <= 0 || B < 0) return TC_ERR_SHAPE;
  for (int t = 0; t < n_tables; t++) {
    if (!LUT[t] || !Idx[t] || !O[t]) return TC_ERR_NULL;
    if (E[t] <= 0 || L[t] <= 0) return TC_ERR_SHAPE;
  }
  for (int t = 0; t < n_tables; t++) {
    if (misaligned(LUT[t]) || misaligned(Idx[t]) || misaligned(O[t])) return TC_ERR_ALIGN;
    for (int m = 0; m < n_tables; m++) {
      if (static_cast<const void*>(O[t]) == LUT[m] || static_cast<const void*>(O[t]) == Idx[m]) return TC_ERR_ALIAS;
      if (m != t && O[t] == O[m]) return TC_ERR_ALIAS;
    }
    if (prod_reaches({std::max<int64_t>(B, 1), L[t]}, kMaxElems) || E[t] > (int64_t)INT32_MAX + 1) return TC_ERR_UNSUPPORTED;
  }
  if (prod_reaches({std::max<int64_t>(B, 1), D}, kMaxElems)) return TC_ERR_UNSUPPORTED;
  if (B == 0) return TC_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  LutArgs a{};
  for (int t = 0; t < n_tables; t++) {
    a.LUT[t] = LUT[t]; a.Idx[t] = Idx[t]; a.O[t] = O[t]; a.E[t] = E[t]; a.L[t] = (int)L[t];
  }
  a.D = (int)D; a.B = (int)B;
  const int v = (D % 4 == 0) ? 4 : 1;
  const int64_t units = D / v;
  int cpw = 1;
  while (cpw < units && cpw < WG_THREADS) cpw *= 2;
  a.cpw = cpw;
  a.blocks = (int)ceil_div(units, cpw);
  const int64_t grid = (int64_t)n_tables * B * a.blocks;
  if (grid > kMaxGrid) return TC_ERR_UNSUPPORTED;
  if (v == 4) lut_sum_kernel<4><<<dim3((unsigned)grid), dim3(WG_THREADS), 0, s>>>(a);
  else lut_sum_kernel<1><<<dim3((unsigned)grid), dim3(WG_THREADS), 0, s>>>(a);
  return took("lut:sum", launch_status());
}

}  // extern "C"
