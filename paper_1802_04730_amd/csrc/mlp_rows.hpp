// Fused chain of fcrelu layers for SMALL batches (Section 3, listing fcrelu;
// appendix "Production Models", listings MLP1 / MLP3; the benchmark's batch of
// 128 through 1024 -> 1024 -> 512 -> 256):
//
//   O_l(b,n) = max(0, bias_l(n) + sum_m In_l(b,m) * W_l(n,m)),   In_{l+1} = O_l
//
// The launch is one workgroup per compute unit, all resident, and a layer's
// 16 x 16 output tiles (row tile = 16 rows of the batch, column tile = 16
// output features) are dealt out so that the WEIGHTS cross the chip's fabric
// once.  The chip is 8 XCDs, each with its own L2 behind a port of about
// 1 TB/s, and the dispatcher deals workgroups to them in turn (measured:
// workgroup w runs on XCD w % 8).  Workgroup w therefore belongs to share
// x = w % 8, and share x owns the column tiles x, x + 8, x + 16, .. of EVERY
// layer, for all row tiles: an XCD pulls one eighth of every weight matrix
// (0.9 MB of the benchmark's 7.3 MB) instead of all of it.  (With one row tile
// per XCD, each XCD pulled every weight; at the port's rate that was 3 us of
// the first layer alone: the same kernel made to fetch only 8 distinct weight
// tiles per XCD, wrong results and all, ran 2.9 us faster.)  What crosses XCDs
// instead is the activations, 1 MB per layer boundary and XCD, served from the
// producers' write-through stores.  (Nothing depends on the placement for correctness:
// all exchange is by agent-scope stores, loads and flags.)
//
// Inside a share the R = gridDim / 8 workgroups take (column tile, row tile)
// jobs: one job each while there are at most R of them (later layers of the
// benchmark), else one column tile with a PAIR of row tiles -- one weight tile
// against two sets of activations, one after the other (first layer).  The
// host checks that a layer never has more than R pairs per share.
//
// One workgroup = 8 wavefronts that split the reduction into 8 contiguous
// slices of K/8 elements.  Operands reach the matrix core like this:
//  - weights (and the caller's fp32 input): a wavefront brings its slice of a
//    16-row tile from global memory STRAIGHT INTO LDS (global_load_lds, 16 bytes
//    per lane, 1 KiB of whole row pieces per instruction: no registers, no LDS
//    write instructions; lane-per-row loads in MFMA layout measured four times
//    slower, 64 separate requests per instruction).  The hardware puts lane i's
//    16 bytes at base + 16 i, so WHICH piece a lane fetches is chosen such that
//    the image is conflict-free for the reads: piece p of row r sits in slot
//    p ^ (r mod pieces) of the row.  A lane then reads row r16, pieces 4j + q,
//    whose elements e = 0..3 feed MFMA step (j, e).  A slice is private to its
//    wavefront, so no wavefront waits for another inside a layer.  The weight
//    tile is read out of LDS into registers once and serves both row tiles of
//    a pair; the second row tile's input follows the first one's through the
//    same LDS slice.  The first layer's operands cannot be requested ahead, so
//    there the slice travels in sub-slices of 32 reduction elements (whole
//    128-byte lines of 8 rows per instruction) and is contracted sub-slice by
//    sub-slice as it lands;
//  - activations between layers: the workspace copy is the library's own, so it
//    is WRITTEN in the layout the next layer reads: [row tile][feature][row]
//    doubles.  A lane's operand for step (j, e) is one 8-byte load, and the 16
//    lanes of a reduction slot read 128 contiguous bytes: no LDS at all on the
//    dependent path.  These loads are agent-scope loads (they never take a stale
//    line from a cache), so the wait needs no cache invalidation: an invalidation
//    by all workgroups at once was measured at 1.7 us per layer boundary.
// The weight tile of layer l+1 is requested as soon as layer l has issued its
// stores and flags (a tile of 32 KB or more: once all wavefronts of the
// workgroup have, so that its requests do not delay their stores'
// acknowledgements) and travels during the hand-over; the wavefronts that do not
// poll turn it into fp64 operands while they wait (on this chip nothing
// overlaps an fp64 MFMA on its SIMD: a conversion costs 8-10 of the MFMA's 64
// clocks wherever it stands).
// The 8 partial tiles are combined through LDS in a fixed order, bias first
// (the listing's first statement); clamp in fp64; O_l leaves as fp32 (if the
// caller wants it) and as fp64 into the workspace.  No activation is rounded
// before it is consumed.
//
// Hand-over between layers, without any read-modify-write and without a
// producer-side workgroup barrier: the wavefront that has written 4 columns of
// a tile of O_l (16 rows, into the workspace) waits for its own stores to be
// acknowledged and then sets the flag word of those 4 columns of that row
// tile; in the next layer one wavefront per workgroup polls the K/4 flag words
// of each row tile it consumes (two 8-byte loads per lane, in flight together)
// while the others meet it at the workgroup barrier.  Flags only ever go from 0
// to 1: workgroup 0 zeroes them and then publishes the call's 64-bit token;
// nobody writes or trusts a flag before it has seen that token; the last
// workgroup out withdraws it, so a replayed HIP graph (same token) starts
// clean.  Every spin is bounded: on expiry the error word is raised and the
// wavefront goes on, so the grid always drains.
//
// Requirements (checked by the host): every reduction extent one of 128, 256,
// 512, 1024; gridDim a multiple of 8; at most gridDim / 8 pairs per share in
// every layer; the flag words fit the sync area.
#pragma once
#include "mlp_fused.hpp"
#include "tc355_device.hpp"

namespace tc355 {

constexpr int MR_WAVES = 8;
constexpr int MR_THREADS = MR_WAVES * WAVE;
constexpr int MR_SHARES = 8;  // shares of the column tiles (= XCDs of the chip)
constexpr int MR_MAXT = 2;    // row tiles per workgroup and layer
constexpr int MR_MAXJ = 8;    // 16-element groups of a wavefront's reduction slice (K / 8 / 16)
constexpr int MR_MAX_WG = 256;
constexpr int MR_SLICE_BYTES = 16 * 128 * 4;                  // a wavefront's slice of a tile: 16 rows x (1024 / 8) fp32
constexpr int MR_AREA_BYTES = MR_WAVES * MR_SLICE_BYTES;       // one 16-row tile of up to 1024 fp32: 64 KiB
constexpr int MR_PART_BYTES = MR_WAVES * MR_MAXT * WAVE * 32;  // the partial tiles
constexpr int MR_LDS_BYTES = 2 * MR_AREA_BYTES + MR_PART_BYTES;  // 160 KiB: one workgroup per compute unit
// flags live behind the header of the sync area: one 32-bit word per 4 output columns of a row tile,
// [boundary][row tile][column / 4], `fstride` words per (boundary, row tile)
constexpr int MR_FLAG_WORD0 = MLP_SYNC_WORDS;

struct MlpRowsArgs {
  const float* I;
  const float* W[MLP_MAX_LAYERS];
  const float* bias[MLP_MAX_LAYERS];
  float* O[MLP_MAX_LAYERS];
  double* act[MLP_MAX_LAYERS];
  unsigned* sync;
  unsigned long long token;
  int dims[MLP_MAX_LAYERS + 1];
  int batch;
  int n_layers;
  int groups;   // number of 16-row tiles of the batch
  int fstride;  // flag words per (boundary, row tile): 4 x the most column tiles of any layer but the last
  unsigned spin_limit;
};

// Host and device: how a layer with CT column tiles and RT row tiles is dealt out inside a share of R workgroups.
// Single jobs while they fit, else pairs of row tiles; `fits` is false if even the pairs do not.
struct MrDeal {
  int per_ct;  // workgroups per column tile of the share (= row tiles, or pairs of them)
  int nrt;     // row tiles per workgroup: 1 or 2
  bool fits;
};
__host__ __device__ inline MrDeal mr_deal(int CT, int RT, int R) {
  const int max_nct = (CT + MR_SHARES - 1) / MR_SHARES, RP = (RT + 1) / 2;
  MrDeal d;
  if (max_nct * RT <= R) { d.per_ct = RT; d.nrt = 1; d.fits = true; }
  else { d.per_ct = RP; d.nrt = 2; d.fits = max_nct * RP <= R; }
  return d;
}

struct MrPlace {
  int lane, wave, r16, q;
  int share, rank, R;  // share of the column tiles (w % 8), this workgroup's number in it, workgroups in it
};

// This workgroup's job in a layer: column tile ct, row tiles rt0 .. rt0 + nrt - 1 (nrt = 0: none).
struct MrJob {
  int ct, rt0, nrt;
};
__device__ __forceinline__ MrJob mr_job(const MrPlace& c, int M, int RT) {
  const int CT = (M + 15) >> 4;
  const MrDeal d = mr_deal(CT, RT, c.R);
  const int i = c.rank / d.per_ct, u = c.rank - i * d.per_ct;
  MrJob j;
  j.ct = c.share + MR_SHARES * i;
  j.rt0 = d.nrt * u;
  j.nrt = j.ct < CT ? max(0, min(d.nrt, RT - j.rt0)) : 0;
  return j;
}

// Index (in doubles) of activation (row r of the tile, feature n) in the workspace copy of a layer of width M.
__device__ __forceinline__ size_t mr_act_index(int rt, int M, int r, int n) { return ((size_t)rt * M + n) * 16 + r; }

// Geometry of a wavefront's slice for a reduction of K in {128, 256, 512, 1024}: ks = K/8 elements per row,
// pieces = ks/4 16-byte pieces per row (a power of two), nj = pieces/4 load instructions and MFMA piece groups.
__device__ __forceinline__ int mr_log2_pieces(int K) { return 31 - __builtin_clz((unsigned)K >> 5); }

// Bring this wavefront's slice of 16 rows (row0 .. row0+15, clamped to last_row) of the row-major fp32 matrix `mat`
// with rows of K elements straight into LDS at `slice`.  Instruction n covers rows n*rpi .. n*rpi + rpi - 1
// (rpi = 64 / pieces); the lane that the hardware places at slot x of row r fetches piece x ^ (r mod pieces).
__device__ __forceinline__ void mr_fetch(const float* mat, int K, int row0, int last_row, const MrPlace& c, char* slice) {
  typedef __attribute__((address_space(1))) const void* gptr;
  typedef __attribute__((address_space(3))) void* lptr;
  const int lp = mr_log2_pieces(K), pieces = 1 << lp, nj = pieces >> 2, ks = K >> 3;
  const int xs = c.lane & (pieces - 1), rl = c.lane >> lp, rpi = WAVE >> lp;
  const float* src0 = mat + (size_t)c.wave * ks;
#pragma unroll
  for (int n = 0; n < MR_MAXJ; n++) {
    if (n < nj) {  // uniform
      const int row = n * rpi + rl;
      const int piece = xs ^ (row & (pieces - 1));
      const float* src = src0 + (size_t)min(row0 + row, last_row) * K + 4 * piece;
      __builtin_amdgcn_global_load_lds((gptr)src, (lptr)(slice + n * 1024), 16, 0, 0);
    }
  }
}

// The same for the first layer, whose operands nobody could request ahead: the slice is cut into sub-slices of 32
// reduction elements (16 rows x 128 bytes, whole cache lines; 2 instructions of 8 rows each), so that the contraction
// starts on sub-slice 0 while the others travel.  Sub-slice g sits at slice + 2048 g (K = 128: one instruction, as
// above); within it, piece p of row r is in slot p ^ (r mod 8) of the row.
__device__ __forceinline__ void mr_fetch_sub(const float* mat, int K, int row0, int last_row, const MrPlace& c, char* slice, int g) {
  typedef __attribute__((address_space(1))) const void* gptr;
  typedef __attribute__((address_space(3))) void* lptr;
  const int lps = min(mr_log2_pieces(K), 3), pieces = 1 << lps, ks = K >> 3;
  const int xs = c.lane & (pieces - 1), rl = c.lane >> lps, rpi = WAVE >> lps, ni = 16 / rpi;
  const float* src0 = mat + (size_t)c.wave * ks + 4 * pieces * g;
#pragma unroll
  for (int n = 0; n < 2; n++) {
    if (n < ni) {  // uniform
      const int row = n * rpi + rl;
      const int piece = xs ^ (row & (pieces - 1));
      const float* src = src0 + (size_t)min(row0 + row, last_row) * K + 4 * piece;
      __builtin_amdgcn_global_load_lds((gptr)src, (lptr)(slice + (g * ni + n) * 1024), 16, 0, 0);
    }
  }
}
__device__ __forceinline__ int mr_subslices(int K) { return max(1, K >> 8); }

// Pieces 4j + q of row r16 of a slice fetched in sub-slices (NJ = K / 128).
template <int NJ>
__device__ __forceinline__ f4 mr_read_sub(const char* slice, const MrPlace& c, int j) {
  int slot;
  if constexpr (NJ == 1) slot = (c.r16 << 2) + (c.q ^ (c.r16 & 3));
  else slot = ((j >> 1) << 7) + (c.r16 << 3) + ((4 * (j & 1) + c.q) ^ (c.r16 & 7));
  return *reinterpret_cast<const f4*>(slice + 16 * slot);
}

template <int N>
__device__ __forceinline__ void mr_wait_vm_c() {
  static_assert(N >= 0 && N < 64, "the counter has 6 bits");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most n of this wavefront's vector-memory operations are outstanding (the counter retires in order).
// The compiler does not order LDS reads after the global_load_lds requests that fill the LDS, so every such
// dependency is stated with this.
__device__ __forceinline__ void mr_wait_vm(int n) {  // n: uniform; rounded down to a count that has an encoding here
  if (n >= 32) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
  else if (n >= 17) asm volatile("s_waitcnt vmcnt(17)" ::: "memory");
  else if (n >= 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else if (n >= 9) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
  else if (n >= 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if (n >= 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
  else if (n >= 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else if (n >= 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
  else if (n >= 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
  else if (n >= 1) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Pieces 4j + q of row r16 of a slice, as the MFMA wants them.
__device__ __forceinline__ f4 mr_read(const char* slice, const MrPlace& c, int lp, int j) {
  const int slot = (c.r16 << lp) + ((4 * j + c.q) ^ (c.r16 & ((1 << lp) - 1)));
  return *reinterpret_cast<const f4*>(slice + 16 * slot);
}

// Workgroup 0 of a chained call: this call's flags start at zero; then the token says so.
__device__ __forceinline__ void mr_publish_token(const MlpRowsArgs& p, unsigned long long* tokp) {
  const int tid = threadIdx.x;
  unsigned* fw = p.sync + MR_FLAG_WORD0;
  const int nwords = (p.n_layers - 1) * p.groups * p.fstride;
  for (int i = tid; i < nwords; i += MR_THREADS) __hip_atomic_store(fw + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (tid == 0) {
    __hip_atomic_store(p.sync + MLP_SYNC_EXIT, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p.sync + MLP_SYNC_ERROR, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // every wavefront's zeroes are acknowledged (a plain wait for everything: the operand requests count too) ...
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();  // ... before the token goes out.  (Relaxed: the zeroes are write-through stores that have been
  // acknowledged; a release here would write back this XCD's whole L2.)
  if (tid == 0) __hip_atomic_store(tokp, p.token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One layer's share of this workgroup: job `jb` (nrt >= 1).  TA is float for the caller's input and double for the
// workspace copy of the previous layer.  `slice`: this wavefront's LDS slice of the layer's weight tile, already
// requested; `ain`: its LDS slice for the input rows (layer 0 only).  `part`: the LDS area for the partial tiles; the
// caller separates layers by a barrier.  NJ = K / 128 is a template parameter: with the trip counts known the
// compiler can count the outstanding loads (behind a branch on a run-time count it waits for all of them before the
// first use of any).
template <typename TA, int NJ>
__device__ __forceinline__ void mr_layer_n(const MlpRowsArgs& p, const MrPlace& c, int l, const MrJob jb,
                                           const TA* __restrict__ Ain, char* slice, char* ain, d4* part,
                                           unsigned long long* tokp, bool& token_seen) {
  constexpr int K = 128 * NJ, ks = K >> 3;
  static_assert(NJ == 1 || NJ == 2 || NJ == 4 || NJ == 8, "reduction extents 128, 256, 512, 1024");
  const int M = p.dims[l + 1];
  const bool two = jb.nrt == 2;  // uniform
  const bool chain = l + 1 < p.n_layers;

  // the bias of this thread's output element (used after the contraction; requested first, lands first).
  // Threads 0..255 finish row tile rt0, threads 256..511 row tile rt0 + 1; thread i of a tile owns the element at
  // position i of the tile's 2 KiB block in the workspace layout, so those stores are contiguous.
  const int fin_t = c.wave >> 2, fin_i = (c.wave & 3) * WAVE + c.lane;
  const int fin_r = fin_i & 15, fin_c = fin_i >> 4;
  const int fin_col = 16 * jb.ct + fin_c;
  const float bias_v = p.bias[l][min(fin_col, M - 1)];

  unsigned long long tok_early = 0;
  d4 acc0 = d4_zero(), acc1 = d4_zero();
  constexpr int lp = NJ == 1 ? 2 : NJ == 2 ? 3 : NJ == 4 ? 4 : 5;
  f4 b[NJ];  // this layer's weight tile, read out of LDS once and used for both row tiles
  if constexpr (sizeof(TA) == 4) {
    // ---- layer 0: the kernel's first instructions requested, sub-slice by sub-slice, the input rows of row tile rt0
    // (into `ain`) and the weight tile (into `slice`); the only younger request is the bias.  Sub-slice g is
    // contracted as soon as it has landed.  With a second row tile, its input is requested into `ain` as soon as the
    // first one has been read out of it, and travels while the first tile is contracted.
    constexpr int NS = NJ <= 2 ? 1 : NJ / 2, JS = NJ / NS, NI = NJ == 1 ? 1 : 2;  // sub-slices, their j's, instructions each
    f4 a[NJ];
#pragma unroll
    for (int g = 0; g < NS; g++) {
      if (g == 0) mr_wait_vm_c<2 * NI * (NS - 1) + 1>();
      else if (g == 1) mr_wait_vm_c<(NS > 1 ? 2 * NI * (NS - 2) : 0) + 1>();
      else if (g == 2) mr_wait_vm_c<(NS > 2 ? 2 * NI * (NS - 3) : 0) + 1>();
      else mr_wait_vm_c<1>();
#pragma unroll
      for (int j = g * JS; j < (g + 1) * JS; j++) {
        a[j] = mr_read_sub<NJ>(ain, c, j);
        b[j] = mr_read_sub<NJ>(slice, c, j);
      }
      if (g == NS - 1) {
        // by now workgroup 0 has long published the token: requested here, looked at after the contraction
        if (chain) tok_early = __hip_atomic_load(tokp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (two) {
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the first input slice has been read out
#pragma unroll
          for (int h = 0; h < NS; h++) mr_fetch_sub(Ain, K, 16 * (jb.rt0 + 1), p.batch - 1, c, ain, h);
        }
      }
#pragma unroll
      for (int j = g * JS; j < (g + 1) * JS; j++)
#pragma unroll
        for (int e = 0; e < 4; e++) acc0 = mfma_f64((double)a[j][e], (double)b[j][e], acc0);
    }
    if (two) {
      mr_wait_vm(0);  // the second row tile's input, requested above, has landed
#pragma unroll
      for (int j = 0; j < NJ; j++) a[j] = mr_read_sub<NJ>(ain, c, j);
#pragma unroll
      for (int j = 0; j < NJ; j++)
#pragma unroll
        for (int e = 0; e < 4; e++) acc1 = mfma_f64((double)a[j][e], (double)b[j][e], acc1);
    }
  } else {
    // ---- later layers: the activations of this wavefront's slice come from the workspace copy, already in MFMA
    // layout (a[j][e] = In[row r16][slice + 16 j + 4 q + e], agent-scope loads: never a stale line from a cache); the
    // weight tile was requested a hand-over ago
    // Wavefront 0 is still polling the flags of the row tile(s); the others turn their weight slice into fp64
    // operands meanwhile (a conversion takes the matrix pipe's time: 8-10 clocks against the MFMA's 64) and meet it at
    // the barrier.
    double bd[NJ][4];
    if (c.wave != 0) {  // uniform per wavefront
      mr_wait_vm(0);    // the weights have landed in LDS
#pragma unroll
      for (int j = 0; j < NJ; j++) {
        b[j] = mr_read(slice, c, lp, j);
#pragma unroll
        for (int e = 0; e < 4; e++) bd[j][e] = (double)b[j][e];
      }
    }
    __syncthreads();  // wavefront 0 has seen the flags (and, if nobody had yet, the token)
    double a[NJ][4];
    {
      const int rows0 = min(16, p.batch - 16 * jb.rt0);
      const double* s0 = Ain + mr_act_index(jb.rt0, K, min(c.r16, rows0 - 1), c.wave * ks + 4 * c.q);
#pragma unroll
      for (int j = 0; j < NJ; j++)
#pragma unroll
        for (int e = 0; e < 4; e++)
          a[j][e] = __hip_atomic_load(s0 + (size_t)(16 * j + e) * 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (c.wave == 0) {
      mr_wait_vm(4 * NJ);  // everything older than these 4 nj loads is done: the weights have landed in LDS
#pragma unroll
      for (int j = 0; j < NJ; j++) {
        b[j] = mr_read(slice, c, lp, j);
#pragma unroll
        for (int e = 0; e < 4; e++) bd[j][e] = (double)b[j][e];
      }
    }
#pragma unroll
    for (int j = 0; j < NJ; j++)
#pragma unroll
      for (int e = 0; e < 4; e++) acc0 = mfma_f64(a[j][e], bd[j][e], acc0);
    if (two) {
      const int rows1 = min(16, p.batch - 16 * (jb.rt0 + 1));
      const double* s1 = Ain + mr_act_index(jb.rt0 + 1, K, min(c.r16, rows1 - 1), c.wave * ks + 4 * c.q);
#pragma unroll
      for (int j = 0; j < NJ; j++)
#pragma unroll
        for (int e = 0; e < 4; e++)
          a[j][e] = __hip_atomic_load(s1 + (size_t)(16 * j + e) * 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
      for (int j = 0; j < NJ; j++)
#pragma unroll
        for (int e = 0; e < 4; e++) acc1 = mfma_f64(a[j][e], bd[j][e], acc1);
    }
  }
  part[(c.wave * MR_MAXT + 0) * WAVE + c.lane] = acc0;
  if (two) part[(c.wave * MR_MAXT + 1) * WAVE + c.lane] = acc1;
  __syncthreads();

  // ---- finish
  const bool fin = fin_t < jb.nrt;  // uniform per wavefront
  double x = (double)bias_v;        // bias first (the listing's first statement), then a fixed order
  if (fin) {
    const int dl = fin_c + 16 * (fin_r & 3), dv = fin_r >> 2;  // where the MFMA result layout keeps it: lane, element
    const double* pd = reinterpret_cast<const double*>(part) + 4 * (fin_t * WAVE + dl) + dv;  // one 8-byte read each
#pragma unroll
    for (int u = 0; u < MR_WAVES; u++) x += pd[4 * u * MR_MAXT * WAVE];
    x = relu64(x);
  }
  __syncthreads();  // the partial tiles have been read: the next layer may overwrite them
  if (fin) {
    const int rt = jb.rt0 + fin_t, row = 16 * rt + fin_r;
    if (row < p.batch && fin_col < M) {
      if (chain) act_store(p.act[l] + mr_act_index(rt, M, fin_r, fin_col), x);
      if (p.O[l]) p.O[l][(size_t)row * M + fin_col] = (float)x;
    }
    if (chain) {
      // This wavefront has just written columns 4u .. 4u+3 (u = wave % 4) of its tile, all 16 rows.  Once its stores
      // are acknowledged (neither a fence of workgroup scope nor a workgroup barrier waits for outstanding global
      // stores on this target), their flag goes out.
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (!token_seen) {  // flags may be written only once workgroup 0 has zeroed them and published the token
        unsigned spins = 0;
        while (tok_early != p.token) {
          __builtin_amdgcn_s_sleep(2);
          if (++spins >= p.spin_limit) {
            if (c.lane == 0) __hip_atomic_store(p.sync + MLP_SYNC_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
          tok_early = __hip_atomic_load(tokp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        token_seen = true;
      }
      unsigned* flags_out = p.sync + MR_FLAG_WORD0 + ((size_t)l * p.groups + rt) * p.fstride;
      if (c.lane == 0)
        __hip_atomic_store(flags_out + 4 * jb.ct + (c.wave & 3), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// WIDE: every reduction extent of the chain is 512 or 1024 (the host says so): the kernel then carries only those two
// layer bodies.  Every instruction of this kernel runs once or a few times per launch, so what it costs to fetch the
// code shows: the benchmark chain runs 0.15 us faster on the smaller kernel.
template <typename TA, bool WIDE>
__device__ __forceinline__ void mr_layer(const MlpRowsArgs& p, const MrPlace& c, int l, const MrJob jb,
                                         const TA* __restrict__ Ain, char* slice, char* ain, d4* part,
                                         unsigned long long* tokp, bool& token_seen) {
  const int nj = p.dims[l] >> 7;  // uniform
  if constexpr (WIDE) {
    if (nj == 4) mr_layer_n<TA, 4>(p, c, l, jb, Ain, slice, ain, part, tokp, token_seen);
    else mr_layer_n<TA, 8>(p, c, l, jb, Ain, slice, ain, part, tokp, token_seen);
  } else {
    switch (nj) {
      case 1: mr_layer_n<TA, 1>(p, c, l, jb, Ain, slice, ain, part, tokp, token_seen); break;
      case 2: mr_layer_n<TA, 2>(p, c, l, jb, Ain, slice, ain, part, tokp, token_seen); break;
      case 4: mr_layer_n<TA, 4>(p, c, l, jb, Ain, slice, ain, part, tokp, token_seen); break;
      default: mr_layer_n<TA, 8>(p, c, l, jb, Ain, slice, ain, part, tokp, token_seen); break;
    }
  }
}

template <bool WIDE>
__global__ __launch_bounds__(MR_THREADS, 1) void mlp_rows_kernel(MlpRowsArgs p) {
  extern __shared__ __attribute__((aligned(32))) char mr_smem[];
  // Everything that the first requests need is read from the argument block in one go: read where it is first
  // used, it is two dependent trips to memory before the first request goes out.
  asm volatile("" ::"s"(p.I), "s"(p.W[0]), "s"(p.dims[0]), "s"(p.dims[1]), "s"(p.batch), "s"(p.groups), "s"(p.n_layers),
               "s"(p.sync));
  const int tid = threadIdx.x;
  MrPlace c;
  c.lane = tid & (WAVE - 1);
  c.wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  c.r16 = c.lane & 15;
  c.q = c.lane >> 4;
  const int nwg = (int)gridDim.x, w = (int)blockIdx.x, RT = p.groups;
  c.share = w % MR_SHARES;
  c.rank = w / MR_SHARES;
  c.R = nwg / MR_SHARES;
  d4* part = reinterpret_cast<d4*>(mr_smem + 2 * MR_AREA_BYTES);
  unsigned long long* tokp = reinterpret_cast<unsigned long long*>(p.sync + MLP_SYNC_TOKEN);
  const bool chained = p.n_layers > 1;
  bool token_seen = !chained;  // per wavefront: has it seen this call's token?

  char* slice0 = mr_smem + c.wave * MR_SLICE_BYTES;                  // this wavefront's slice of the weight tile
  char* slice1 = mr_smem + MR_AREA_BYTES + c.wave * MR_SLICE_BYTES;  // layer 0: its slice of the input row tile(s)

  MrJob jb = mr_job(c, p.dims[1], RT);
  // the input rows and the weight tile of the first layer's job are requested before anything else
  if (jb.nrt > 0) {  // uniform
    const int ns = mr_subslices(p.dims[0]);
#pragma unroll
    for (int g = 0; g < 4; g++) {
      if (g < ns) {  // uniform
        mr_fetch_sub(p.I, p.dims[0], 16 * jb.rt0, p.batch - 1, c, slice1, g);
        mr_fetch_sub(p.W[0], p.dims[0], 16 * jb.ct, p.dims[1] - 1, c, slice0, g);
      }
    }
  }
  if (chained && w == 0) mr_publish_token(p, tokp);  // (workgroup 0 always has a job in layer 0: it waits for its requests here)

  for (int l = 0; l < p.n_layers; l++) {
    MrJob jn{0, 0, 0};
    if (l + 1 < p.n_layers) jn = mr_job(c, p.dims[l + 2], RT);
    if (jb.nrt == 0) {
      // no job in this layer
    } else if (l == 0) {
      mr_layer<float, WIDE>(p, c, 0, jb, p.I, slice0, slice1, part, tokp, token_seen);
    } else {
      // Layer l reads row tiles rt0 .. of O_{l-1}: a row tile is all there once the K/4 flag words of boundary l-1
      // are set.  One wavefront polls them (two 8-byte loads per lane and row tile, in flight together), the others
      // wait at the workgroup barrier: eight polling wavefronts per workgroup were measured slower.
      if (c.wave == 0) {
        unsigned spins = 0;
        bool ok = true;
        if (!token_seen) {  // a workgroup without a job in the first layer comes here first
          while (__hip_atomic_load(tokp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.token) {
            __builtin_amdgcn_s_sleep(2);
            if (++spins >= p.spin_limit) { ok = false; break; }
          }
        }
        const int npairs = p.dims[l] >> 3;  // K/4 flag words (32 .. 256), two to a load
        const unsigned long long* fin0 =
            reinterpret_cast<const unsigned long long*>(p.sync + MR_FLAG_WORD0 + ((size_t)(l - 1) * RT + jb.rt0) * p.fstride);
        const unsigned long long* fin1 =
            reinterpret_cast<const unsigned long long*>(p.sync + MR_FLAG_WORD0 + ((size_t)(l - 1) * RT + jb.rt0 + jb.nrt - 1) * p.fstride);
        const int i0 = min(c.lane, npairs - 1), i1 = min(c.lane + WAVE, npairs - 1);
        const unsigned long long want = 0x0000000100000001ull;
        while (ok) {
          if (spins >= p.spin_limit) {  // (a limit of 0: gives up without looking)
            ok = false;
            break;
          }
          const unsigned long long v0 = __hip_atomic_load(fin0 + i0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned long long v1 = __hip_atomic_load(fin0 + i1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned long long v2 = __hip_atomic_load(fin1 + i0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned long long v3 = __hip_atomic_load(fin1 + i1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (__builtin_amdgcn_ballot_w64(v0 != want || v1 != want || v2 != want || v3 != want) == 0) break;
          __builtin_amdgcn_s_sleep(1);
          ++spins;
        }
        if (!ok && c.lane == 0) __hip_atomic_store(p.sync + MLP_SYNC_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      token_seen = true;  // (for the other wavefronts: by the barrier at which the layer meets wavefront 0)
      mr_layer<double, WIDE>(p, c, l, jb, p.act[l - 1], slice0, slice1, part, tokp, token_seen);
    }
    // The next layer's weight tile is requested as soon as this layer has issued its stores and flags: it travels
    // while the next layer's wavefronts wait for their activations.
    if (jn.nrt > 0) {
      // A large tile's requests wait until every wavefront of the workgroup has its flag out: the wavefronts that
      // finish no outputs would otherwise start 32 KB of requests while the others' stores still wait for their
      // acknowledgements (benchmark chain 20.2 -> 19.9 us; chains of 128-wide layers lose 0.6 us with it).
      if (p.dims[l + 1] >= 512) __syncthreads();  // uniform
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wavefront has read everything out of its slice
      mr_fetch(p.W[l + 1], p.dims[l + 1], 16 * jn.ct, p.dims[l + 2] - 1, c, slice0);
    }
    jb = jn;
  }

  // The last workgroup out withdraws the token: a replay of a captured HIP graph launches this kernel again with
  // the SAME token, and must again wait for workgroup 0 to zero the flags.  Nobody counts itself out before it has
  // seen the token: workgroup 0 zeroes the counter before it publishes the token, and a workgroup with nothing to do
  // would otherwise get here first and have its count wiped.
  if (chained && tid == 0) {
    if (!token_seen) {
      unsigned spins = 0;
      while (__hip_atomic_load(tokp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.token) {
        __builtin_amdgcn_s_sleep(8);
        if (++spins >= p.spin_limit) {
          __hip_atomic_store(p.sync + MLP_SYNC_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
      }
    }
    const unsigned old = __hip_atomic_fetch_add(p.sync + MLP_SYNC_EXIT, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (unsigned)nwg - 1) __hip_atomic_store(tokp, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

}  // namespace tc355
