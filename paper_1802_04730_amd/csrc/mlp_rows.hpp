// Fused chain of fcrelu layers for SMALL batches (Section 3, listing fcrelu;
// appendix "Production Models", listings MLP1 / MLP3; the benchmark's batch of
// 128 through 1024 -> 1024 -> 512 -> 256):
//
//   O_l(b,n) = max(0, bias_l(n) + sum_m In_l(b,m) * W_l(n,m)),   In_{l+1} = O_l
//
// Row b of O_{l+1} needs row b of O_l and nothing else of it.  So the batch is
// cut into tiles of 16 rows and a GROUP of workgroups takes one row tile through
// ALL layers: only the workgroups of a group ever exchange activations, and only
// they wait for each other between layers.  Workgroup w belongs to group
// w % groups; with 8 row tiles on an 8-XCD chip, whose dispatcher deals
// workgroups to the XCDs in turn (measured: workgroup w runs on XCD w % 8), a
// group is one XCD: the activations never leave that XCD's L2 and a wait
// involves 32 workgroups instead of 256.  (Nothing depends on that placement
// for correctness: data is exchanged with agent-scope write-through stores,
// agent-scope loads and flags, wherever the workgroups run.)  The price: every
// group reads every weight once, 8 x 6.8 MB for the benchmark instead of 1 x --
// but weights depend on no activation, so they are requested a whole wait ahead.
//
// One workgroup = 8 wavefronts on one compute unit.  In layer l it owns the
// column tiles rank, rank + gsize (at most 2) of its row tile; its 8 wavefronts
// split the reduction into 8 contiguous slices of K/8 elements.  Operands reach
// the matrix core like this:
//  - weights (and the caller's fp32 input): a wavefront brings its slice of a
//    16-row tile from global memory STRAIGHT INTO LDS (global_load_lds, 16 bytes
//    per lane, 1 KiB of whole row pieces per instruction: no registers, no LDS
//    write instructions; lane-per-row loads in MFMA layout measured four times
//    slower, 64 separate requests per instruction).  The hardware puts lane i's
//    16 bytes at base + 16 i, so WHICH piece a lane fetches is chosen such that
//    the image is conflict-free for the reads: piece p of row r sits in slot
//    p ^ (r mod pieces) of the row.  A lane then reads row r16, pieces 4j + q,
//    whose elements e = 0..3 feed MFMA step (j, e).  A slice is private to its
//    wavefront, so no wavefront waits for another inside a layer;
//  - activations between layers: the workspace copy is the library's own, so it
//    is WRITTEN in the layout the next layer reads: [row tile][feature][row]
//    doubles.  A lane's operand for step (j, e) is one 8-byte load, and the 16
//    lanes of a reduction slot read 128 contiguous bytes: no LDS at all on the
//    dependent path.  These loads are agent-scope loads (they never take a stale
//    line from a cache), so the wait needs no cache invalidation: an invalidation
//    by all workgroups at once was measured at 1.7 us per layer boundary.
// The weights of layer l+1 are requested as soon as layer l has issued its
// stores and travel during the group's wait.  The 8 partial tiles are combined
// through LDS in a fixed order, bias first (the listing's first statement);
// clamp in fp64; O_l leaves as fp32 (if the caller wants it) and as fp64 into
// the workspace.  No activation is rounded before it is consumed.
//
// Hand-over between layers, without any read-modify-write and without a
// producer-side workgroup barrier: the wavefront that has written 4 columns of
// a tile of O_l (16 rows, into the workspace) waits for its own stores to be
// acknowledged and then sets the flag word of those 4 columns; in the next
// layer one wavefront per workgroup polls the K/4 flag words of its row tile
// (at most 256: two 8-byte loads per lane, in flight together) while the
// others wait at the workgroup barrier.  Flags only ever go from 0 to 1: workgroup 0 zeroes them
// and then publishes the call's 64-bit token; nobody writes or trusts a flag
// before it has seen that token (requested while the first layer's operands
// arrive, checked before the first flag is written or read); the last
// workgroup out withdraws it, so a replayed HIP graph (same token) starts
// clean.  Every spin is bounded: on expiry the error word is raised and the
// wavefront goes on, so the grid always drains.
//
// Requirements (checked by the host): every reduction extent one of 128, 256,
// 512, 1024; at most 2 column tiles per workgroup in every layer.
#pragma once
#include "mlp_fused.hpp"
#include "tc355_device.hpp"

namespace tc355 {

constexpr int MR_WAVES = 8;
constexpr int MR_THREADS = MR_WAVES * WAVE;
constexpr int MR_MAXT = 2;    // column tiles per workgroup and layer
constexpr int MR_MAXJ = 8;    // 16-element pieces of a wavefront's reduction slice (K / 8 / 16)
constexpr int MR_MAX_WG = 256;
constexpr int MR_SLICE_BYTES = 16 * 128 * 4;                  // a wavefront's slice of a tile: 16 rows x (1024 / 8) fp32
constexpr int MR_AREA_BYTES = MR_WAVES * MR_SLICE_BYTES;       // one 16-row tile of up to 1024 fp32: 64 KiB
constexpr int MR_PART_BYTES = MR_WAVES * MR_MAXT * WAVE * 32;  // the partial tiles
constexpr int MR_LDS_BYTES = MR_MAXT * MR_AREA_BYTES + MR_PART_BYTES;  // 160 KiB: one workgroup per compute unit
// flags live behind the header of the sync area: one 32-bit word per 4 output columns of a row tile,
// [boundary][group][column / 4], with room for MR_MAXT tiles per workgroup
constexpr int MR_FLAG_WORD0 = MLP_SYNC_WORDS;
// words of flags that a chain needs (the host checks that they fit the sync area)
inline int64_t mr_flag_words(int n_layers, int64_t groups, int64_t nwg) {
  return (int64_t)(n_layers - 1) * groups * 4 * MR_MAXT * ((nwg + groups - 1) / groups);
}

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
  int groups;  // number of 16-row tiles of the batch
  unsigned spin_limit;
};

struct MrPlace {
  int lane, wave, r16, q;
  int g, rank, gsize;  // group (= row tile), this workgroup's number in it, workgroups in it
};

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

// One layer's share of this workgroup.  TA is float for the caller's input (its slice is already on its way into
// `slice1`) and double for the workspace copy of the previous layer (read in place).  The first tile's weights are
// on their way into `slice0`; the second tile's into `slice1` (layer 0: requested here, once the input has been
// read out of it).  `part`: the LDS area for the partial tiles; the caller separates layers by a barrier.
// NJ = K / 128 (1, 2, 4 or 8) is a template parameter: with the trip counts known the compiler can count the
// outstanding loads (behind a branch on a run-time count it waits for all of them before the first use of any).
template <typename TA, int NJ>
__device__ __forceinline__ void mr_layer_n(const MlpRowsArgs& p, const MrPlace& c, int l, const TA* __restrict__ Ain,
                                           char* slice0, char* slice1, d4* part, unsigned* flags_out,
                                           const unsigned long long* tokp, bool& token_seen) {
  constexpr int K = 128 * NJ, ks = K >> 3, nj = NJ, lp = NJ == 1 ? 2 : NJ == 2 ? 3 : NJ == 4 ? 4 : 5;
  static_assert(NJ == 1 || NJ == 2 || NJ == 4 || NJ == 8, "reduction extents 128, 256, 512, 1024");
  const int M = p.dims[l + 1];
  const int CT = (M + 15) >> 4;
  if (c.rank >= CT) return;  // uniform: no tile in this layer
  const bool two = c.rank + c.gsize < CT;  // uniform: a second tile
  const int rows = min(16, p.batch - 16 * c.g);  // rows of this row tile inside the batch

  // ---- activations of this wavefront's slice as MFMA A operands: a[j].e[e] = In[row r16][slice + 16j + 4q + e]
  unsigned long long tok_early = 0;
  Vec<TA, 4> a[MR_MAXJ];
  if constexpr (sizeof(TA) == 4) {
    mr_wait_vm(0);  // the input slice (and the first tile's weights) have landed in LDS
    // by now workgroup 0 has long published the token: requested here, looked at after the contraction
    if (p.n_layers > 1) tok_early = __hip_atomic_load(tokp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int j = 0; j < MR_MAXJ; j++) {
      if (j < nj) {
        const f4 t = mr_read(slice1, c, lp, j);
        a[j].e[0] = t[0]; a[j].e[1] = t[1]; a[j].e[2] = t[2]; a[j].e[3] = t[3];
      }
    }
  } else {
    const double* src = Ain + mr_act_index(c.g, K, min(c.r16, rows - 1), c.wave * ks + 4 * c.q);
#pragma unroll
    for (int j = 0; j < MR_MAXJ; j++) {
      if (j < nj) {
#pragma unroll
        for (int e = 0; e < 4; e++)
          a[j].e[e] = __hip_atomic_load(src + (size_t)(16 * j + e) * 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    mr_wait_vm(4 * nj);  // everything older than these 4 nj loads is done: the weights have landed in LDS
  }
  // the bias of this thread's output element (used after the contraction; requested now)
  const int fin_t = c.wave >> 2, fin_i = (c.wave & 3) * WAVE + c.lane;
  const int fin_r = fin_i & 15, fin_c = fin_i >> 4;  // row and column inside the tile: the workspace block's order
  const int fin_col = 16 * (c.rank + fin_t * c.gsize) + fin_c;
  const float bias_v = p.bias[l][min(fin_col, M - 1)];

  // ---- first tile: its weights into registers, then (layer 0) the second tile's weights are requested into the
  // slice that held the input, and travel while the first tile is contracted
  f4 b[MR_MAXJ];
#pragma unroll
  for (int j = 0; j < MR_MAXJ; j++)
    if (j < nj) b[j] = mr_read(slice0, c, lp, j);
  if constexpr (sizeof(TA) == 4) {
    if (two) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the input has been read out of slice1
      mr_fetch(p.W[l], K, 16 * (c.rank + c.gsize), M - 1, c, slice1);
    }
  }
  d4 acc0 = d4_zero(), acc1 = d4_zero();
#pragma unroll
  for (int j = 0; j < MR_MAXJ; j++) {
    if (j < nj) {
#pragma unroll
      for (int e = 0; e < 4; e++) acc0 = mfma_f64((double)a[j].e[e], (double)b[j][e], acc0);
    }
  }
  part[(c.wave * MR_MAXT + 0) * WAVE + c.lane] = acc0;
  if (two) {
    if constexpr (sizeof(TA) == 4) mr_wait_vm(0);  // the second tile's weights, requested above, have landed
#pragma unroll
    for (int j = 0; j < MR_MAXJ; j++)
      if (j < nj) b[j] = mr_read(slice1, c, lp, j);
#pragma unroll
    for (int j = 0; j < MR_MAXJ; j++) {
      if (j < nj) {
#pragma unroll
        for (int e = 0; e < 4; e++) acc1 = mfma_f64((double)a[j].e[e], (double)b[j][e], acc1);
      }
    }
    part[(c.wave * MR_MAXT + 1) * WAVE + c.lane] = acc1;
  }
  __syncthreads();

  // ---- finish: threads 0..255 take tile 0, threads 256..511 tile 1.  Thread i of a tile owns the element that sits
  // at position i of the tile's 2 KiB block in the workspace layout, so those stores are contiguous.
  const bool fin = fin_t == 0 || two;  // uniform per wavefront
  double x = (double)bias_v;  // bias first (the listing's first statement), then a fixed order
  if (fin) {
    const int dl = fin_c + 16 * (fin_r & 3), dv = fin_r >> 2;  // where the MFMA result layout keeps it: lane, element
#pragma unroll
    for (int u = 0; u < MR_WAVES; u++) x += part[(u * MR_MAXT + fin_t) * WAVE + dl][dv];
    x = relu64(x);
  }
  __syncthreads();  // the partial tiles have been read: the next layer may overwrite them
  if (fin) {
    const int row = 16 * c.g + fin_r;
    if (row < p.batch && fin_col < M) {
      if (l + 1 < p.n_layers) act_store(p.act[l] + mr_act_index(c.g, M, fin_r, fin_col), x);
      if (p.O[l]) p.O[l][(size_t)row * M + fin_col] = (float)x;
    }
    if (l + 1 < p.n_layers) {
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
      if (c.lane == 0)
        __hip_atomic_store(flags_out + 4 * (c.rank + fin_t * c.gsize) + (c.wave & 3), 1u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

template <typename TA>
__device__ __forceinline__ void mr_layer(const MlpRowsArgs& p, const MrPlace& c, int l, const TA* __restrict__ Ain,
                                         char* slice0, char* slice1, d4* part, unsigned* flags_out,
                                         const unsigned long long* tokp, bool& token_seen) {
  switch (p.dims[l] >> 7) {  // uniform
    case 1: mr_layer_n<TA, 1>(p, c, l, Ain, slice0, slice1, part, flags_out, tokp, token_seen); break;
    case 2: mr_layer_n<TA, 2>(p, c, l, Ain, slice0, slice1, part, flags_out, tokp, token_seen); break;
    case 4: mr_layer_n<TA, 4>(p, c, l, Ain, slice0, slice1, part, flags_out, tokp, token_seen); break;
    default: mr_layer_n<TA, 8>(p, c, l, Ain, slice0, slice1, part, flags_out, tokp, token_seen); break;
  }
}

__global__ __launch_bounds__(MR_THREADS, 1) void mlp_rows_kernel(MlpRowsArgs p) {
  extern __shared__ __attribute__((aligned(32))) char mr_smem[];
  const int tid = threadIdx.x;
  MrPlace c;
  c.lane = tid & (WAVE - 1);
  c.wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
  c.r16 = c.lane & 15;
  c.q = c.lane >> 4;
  char* slice0 = mr_smem + c.wave * MR_SLICE_BYTES;
  char* slice1 = mr_smem + MR_AREA_BYTES + c.wave * MR_SLICE_BYTES;
  d4* part = reinterpret_cast<d4*>(mr_smem + MR_MAXT * MR_AREA_BYTES);
  const int nwg = (int)gridDim.x, G = p.groups;
  const int w = (int)blockIdx.x;
  c.g = w % G;
  c.rank = w / G;
  c.gsize = (nwg - c.g + G - 1) / G;
  const int fstride = 4 * MR_MAXT * ((nwg + G - 1) / G);  // flag words reserved per group and boundary
  unsigned* flags = p.sync + MR_FLAG_WORD0;
  unsigned long long* tokp = reinterpret_cast<unsigned long long*>(p.sync + MLP_SYNC_TOKEN);
  const bool chained = p.n_layers > 1;

  // the input and the first tile of the first layer's weights are requested before anything else
  if (c.rank < ((p.dims[1] + 15) >> 4)) {  // uniform
    mr_fetch(p.I, p.dims[0], 16 * c.g, p.batch - 1, c, slice1);
    mr_fetch(p.W[0], p.dims[0], 16 * c.rank, p.dims[1] - 1, c, slice0);
  }

  if (chained && w == 0) {
    // this call's flags start at zero; then the token says so
    unsigned* fw = p.sync + MR_FLAG_WORD0;
    const int nwords = (p.n_layers - 1) * G * fstride;
    for (int i = tid; i < nwords; i += MR_THREADS) __hip_atomic_store(fw + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) {
      __hip_atomic_store(p.sync + MLP_SYNC_EXIT, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(p.sync + MLP_SYNC_ERROR, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // every wavefront's zeroes are acknowledged (a plain wait for everything: the requests above count too) ...
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // ... before the token goes out.  (Relaxed: the zeroes are write-through stores that have been
    // acknowledged; a release here would write back this XCD's whole L2.)
    if (tid == 0) __hip_atomic_store(tokp, p.token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  bool token_seen = !chained;  // per wavefront: has it seen this call's token?

  // A layer's weights are requested as soon as the layer before it has issued its stores and flags: they travel
  // while the next layer's wavefronts wait for their activations.
  for (int l = 0; l < p.n_layers; l++) {
    unsigned* fout = flags + ((size_t)l * G + c.g) * fstride;  // boundary l: what layer l writes
    if (l == 0) {
      mr_layer<float>(p, c, 0, p.I, slice0, slice1, part, fout, tokp, token_seen);
    } else {
      // Layer l reads row tile g of O_{l-1}: all of it is there once the K/4 flag bytes of boundary l-1 are set.
      // One wavefront polls them (4 per lane: one load), the others wait at the workgroup barrier: eight polling
      // wavefronts per workgroup were measured slower (their loads delay the flags they wait for).
      if (c.wave == 0 && c.rank < ((p.dims[l + 1] + 15) >> 4)) {
        unsigned spins = 0;
        bool ok = true;
        if (!token_seen) {  // a workgroup without a tile in the first layer comes here first
          while (__hip_atomic_load(tokp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.token) {
            __builtin_amdgcn_s_sleep(2);
            if (++spins >= p.spin_limit) { ok = false; break; }
          }
        }
        // K/4 flag words (32 .. 256): a lane takes up to four of them, as two 8-byte loads that travel together
        const unsigned long long* fin = reinterpret_cast<const unsigned long long*>(flags + ((size_t)(l - 1) * G + c.g) * fstride);
        const int npairs = p.dims[l] >> 3;
        const unsigned long long* f0 = fin + min(c.lane, npairs - 1);
        const unsigned long long* f1 = fin + min(c.lane + WAVE, npairs - 1);
        const unsigned long long want = 0x0000000100000001ull;
        for (;;) {
          const unsigned long long v0 = __hip_atomic_load(f0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          const unsigned long long v1 = __hip_atomic_load(f1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (__builtin_amdgcn_ballot_w64(v0 != want || v1 != want) == 0) break;
          __builtin_amdgcn_s_sleep(1);
          if (++spins >= p.spin_limit) { ok = false; break; }
        }
        if (!ok && c.lane == 0) __hip_atomic_store(p.sync + MLP_SYNC_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (c.rank < ((p.dims[l + 1] + 15) >> 4)) token_seen = true;  // (for the other wavefronts: by the barrier below)
      __syncthreads();
      mr_layer<double>(p, c, l, p.act[l - 1], slice0, slice1, part, fout, tokp, token_seen);
    }
    if (l + 1 < p.n_layers) {
      const int Kn = p.dims[l + 1], Mn = p.dims[l + 2];
      const int CTn = (Mn + 15) >> 4;
      // this wavefront has read everything it needs out of its slices (the contraction consumed it)
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (c.rank < CTn) mr_fetch(p.W[l + 1], Kn, 16 * c.rank, Mn - 1, c, slice0);
      if (c.rank + c.gsize < CTn) mr_fetch(p.W[l + 1], Kn, 16 * (c.rank + c.gsize), Mn - 1, c, slice1);
    }
  }

  // The last workgroup out withdraws the token: a replay of a captured HIP graph launches this kernel again with
  // the SAME token, and must again wait for workgroup 0 to zero the flags.
  // Nobody counts itself out before it has seen the token: workgroup 0 zeroes the counter before it publishes the
  // token, and a workgroup with nothing to do would otherwise get here first and have its count wiped (the token
  // would then survive the launch, and a replay would trust flags that workgroup 0 is about to zero).
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
