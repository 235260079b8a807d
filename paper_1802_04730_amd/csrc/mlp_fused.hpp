// Fused chain of fcrelu layers in ONE kernel launch (Section 3, listing fcrelu;
// appendix "Production Models", listing MLP3: the point of the paper's MLP3 is
// a single kernel for the whole chain).
//
//   O_l(b,n) = max(0, bias_l(n) + sum_m In_l(b,m) * W_l(n,m)),   In_{l+1} = O_l
//
// Persistent kernel: one workgroup of two teams of 4 wavefronts per compute unit (two
// teams, so that one's loads and LDS staging overlap the other's MFMAs) stays
// resident for all layers.  Within a layer, a team takes 16x16 output tiles round-robin;
// its 4 wavefronts each fetch (16-byte loads kept several chunks ahead), stage in
// LDS and contract a quarter of every chunk on the fp64 MFMA; the partial tiles are combined through LDS in a fixed
// order, starting from the bias (the listing's first statement); the clamp is
// applied in fp64 in registers;
// O_l is written as fp32 (if the caller wants it) and as fp64 into the
// workspace, where the next layer reads it after a device-wide barrier.  No
// activation is ever rounded before it is consumed.
//
// The device-wide barrier is an arrival counter in the workspace (one per layer
// boundary).  The fp64 activations are stored and loaded with agent-scope
// accesses, which bypass the per-XCD L2 caches, so the barrier needs no
// whole-cache write-back or invalidate (with 256 workgroups those serialise
// and cost tens of microseconds).  The
// workspace may hold anything on entry: workgroup 0 zeroes the counters when the
// kernel starts and then publishes the call's 64-bit token (unique per call,
// chosen by the host); a workgroup adds itself to a counter only after it has
// seen that token, which by the time a layer is finished is long there; release
// words are compared with the token, so stale ones never match; the last
// workgroup to leave withdraws the token, which makes replays of a captured graph
// (same token every time) safe.  Every
// spin is bounded: if a wait does not end (workgroups not co-resident), the
// waiting workgroup raises the error word and goes on, so the grid always
// drains.
#pragma once
#include "gemm_wave.hpp"
#include "tc355_device.hpp"

namespace tc355 {

constexpr int MLP_MAX_LAYERS = 8;
constexpr int MLP_SYNC_WORDS = 64;  // header of the sync area: token, error word
constexpr int MLP_SYNC_TOKEN = 16;  // words 16,17: token of the call that owns the counters
constexpr int MLP_SYNC_EXIT = 32;   // workgroups that have left the kernel
constexpr int MLP_SYNC_ERROR = 33;  // 1 if a device-wide wait of the last call gave up

struct MlpArgs {
  const float* I;
  const float* W[MLP_MAX_LAYERS];
  const float* bias[MLP_MAX_LAYERS];
  float* O[MLP_MAX_LAYERS];     // fp32 outputs, entries may be nullptr except the last
  double* act[MLP_MAX_LAYERS];  // fp64 copy of O_l for l < n_layers-1
  unsigned* sync;               // MLP_SYNC_WORDS words at the start of the workspace
  unsigned long long token;     // unique per call
  int dims[MLP_MAX_LAYERS + 1];
  int batch;
  int n_layers;
  unsigned spin_limit;
};

// Device-wide barrier, built as a two-level tree so that no address sees more
// than MLP_FANIN arrivals or pollers (hundreds of device-scope atomics on one
// word serialise at the memory side and cost ~10 us).  Workgroup w belongs to
// group w / MLP_FANIN; the last arriver of a group reports to the root counter,
// the last arriver at the root writes the call's token into every group's
// release word, and each workgroup polls only its own group's word.
//
// Memory visibility: the fp64 activations are STORED with agent-scope (sc1)
// write-through accesses, so once every wavefront has waited for its own stores
// (s_waitcnt vmcnt(0): stores count there on this target) and the wavefronts
// have met at __syncthreads(), there is nothing left to write back; after the wait,
// one agent-scope acquire per workgroup drops stale lines from the caches this
// workgroup reads through, and the activations are then LOADED with ordinary
// cached 16-byte loads.  (A whole-cache write-back per workgroup, which a
// release fence would add, was measured at >20 us with 256 workgroups.)
constexpr int MLP_FANIN = 16;
// word layout of one barrier's block inside the sync area (MLP_BAR_WORDS words per layer boundary):
//   [0]                      root counter
//   [16 + 16*g]              arrival counter of group g      (one 64-byte line each)
//   [16 + 16*MLP_GROUPS + 16*g]  release word of group g (low 32 bits of the token)
constexpr int MLP_GROUPS = 64;  // supports up to 1024 workgroups
constexpr int MLP_BAR_WORDS = 16 + 32 * MLP_GROUPS;

__device__ __forceinline__ void mlp_grid_barrier(unsigned* sync, int which, unsigned long long token, unsigned nwg,
                                                 unsigned spin_limit) {
  // Every wavefront first waits until its own vector-memory operations, the write-through activation stores
  // included, have been acknowledged: neither a workgroup-scope release nor the workgroup barrier waits for
  // outstanding global stores on this target, and the arrival below must not overtake them.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();  // now all of this workgroup's write-through stores are acknowledged
  if (threadIdx.x == 0) {
    unsigned* bar = sync + MLP_SYNC_WORDS + which * MLP_BAR_WORDS;
    unsigned* err = sync + MLP_SYNC_ERROR;
    const unsigned long long* tok = reinterpret_cast<const unsigned long long*>(sync + MLP_SYNC_TOKEN);
    const unsigned g = blockIdx.x / MLP_FANIN;
    const unsigned ngroups = (nwg + MLP_FANIN - 1) / MLP_FANIN;
    const unsigned gsize = min((unsigned)MLP_FANIN, nwg - g * MLP_FANIN);
    const unsigned want = (unsigned)token;
    unsigned spins = 0;
    bool ok = true;
    // the counters are valid only once workgroup 0 has published this call's token
    while (__hip_atomic_load(tok, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != token) {
      __builtin_amdgcn_s_sleep(2);
      if (++spins >= spin_limit) { ok = false; break; }
    }
    if (__hip_atomic_fetch_add(bar + 16 + 16 * g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gsize - 1) {
      if (__hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ngroups - 1) {
        for (unsigned i = 0; i < ngroups; i++)
          __hip_atomic_store(bar + 16 + 16 * MLP_GROUPS + 16 * i, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    const unsigned* rel = bar + 16 + 16 * MLP_GROUPS + 16 * g;
    while (ok && __hip_atomic_load(rel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != want) {
      __builtin_amdgcn_s_sleep(2);
      if (++spins >= spin_limit) { ok = false; break; }
    }
    if (!ok) __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // invalidate only; nothing of ours is dirty
  }
  __syncthreads();
}

// fp64 activations cross XCDs inside one kernel: agent-scope write-through stores put
// them where every XCD can fetch them.
__device__ __forceinline__ void act_store(double* p, double x) {
  __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS geometry of one staged chunk of KC reduction elements of a 16-row operand
// tile.  Row strides are padded so that the 16 lanes that share a k slot read 64
// distinct banks with one 16-byte LDS read each.
constexpr int MLP_KC = 128;                  // reduction elements per staged chunk
constexpr int MLP_RS_F = MLP_KC + 4;         // fp32 row stride (words):   = 4 (mod 64)
constexpr int MLP_RS_D = MLP_KC + 2;         // fp64 row stride (doubles): = 2 (mod 32)
constexpr int MLP_BUF_BYTES = 16 * MLP_RS_D * 8 + 16 * MLP_RS_F * 4;  // A (worst case fp64) + B
constexpr int MLP_LDS_BYTES = 2 * MLP_BUF_BYTES + 2 * WAVES_PER_WG * WAVE * 32;  // 2 stages + 2 partial-tile areas

// One layer's share of this workgroup.  TA is float for the first layer (the
// caller's input) and double afterwards (the workspace copy of the previous layer).
//
// The workgroup sees its work as one stream of chunks (KC reduction elements of
// a 16x16 output tile) that runs across its tiles.  Each wavefront owns a quarter
// of every chunk: it fetches that quarter with 16-byte loads (8 or 4 rows of
// 128 contiguous bytes per instruction), NR chunks ahead of the MFMAs through a
// register ring, also across tile boundaries, passes it through its own part of a
// double-buffered LDS stage (which turns row-major 16-byte pieces into MFMA
// operands) and contracts it; the wavefronts meet only at the end of a tile.
// FC: the fcrelu epilogue (sum started from the bias, clamp); without it the body is a plain contraction
// C = A * Wl^T (the transposed matmul of Section 7 at sizes too small for the 64 x 64 block kernel).
template <typename TA, bool FC = true>
__device__ __forceinline__ void mlp_layer(const TA* __restrict__ A, const float* __restrict__ Wl,
                                          const float* __restrict__ bias, float* __restrict__ O,
                                          double* __restrict__ act, int batch, int K, int M, char* smem,
                                          int vwg, int vstep, int team0_jobs_if_team1) {
  // vwg / vstep: this team's number among all teams of the grid and their count (a "team" = 4 wavefronts that own
  // a tile together; a workgroup holds one or two); team0_jobs_if_team1: for the second team of a workgroup, the
  // number of tiles its first team has in this layer (both must pass the same number of barriers), else -1
  constexpr bool A64 = sizeof(TA) == 8;
  constexpr int KC = MLP_KC, NR = 4;
  constexpr int RSA = A64 ? MLP_RS_D : MLP_RS_F;  // row stride of the A stage, in elements of TA
  constexpr int AV = A64 ? 2 : 4;                 // elements of TA per 16-byte load
  constexpr int A_LOADS = 16 * KC / AV / WG_THREADS;  // 16-byte loads per thread and chunk: 4 (fp32) or 8 (fp64)
  constexpr int B_LOADS = 16 * KC / 4 / WG_THREADS;   // 4
  const int tid = threadIdx.x & (WG_THREADS - 1);  // within the team
  const int lane = tid & (WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);  // wavefront-uniform, kept in a scalar register
  const int r16 = lane & 15, q = lane >> 4;
  const int tiles_n = (batch + 15) / 16, tiles_m = (M + 15) / 16;
  const int njobs = tiles_n * tiles_m;
  const int nck = (K + KC - 1) / KC;  // chunks per tile
  const int step = vstep;
  d4* part_base = reinterpret_cast<d4*>(smem + 2 * MLP_BUF_BYTES);
  int parity = 0;  // partial-tile area alternates per tile, so a fast wavefront cannot overwrite one still being read

  struct Regs {
    Vec<TA, AV> a[A_LOADS];
    Vec<float, 4> b[B_LOADS];
  };
  // Position of this thread's 16-byte units inside a 16 x KC operand chunk (same for every chunk).
  constexpr int A_UPR = KC / AV, B_UPR = KC / 4;  // units per row
  // Each wavefront fetches and stages exactly the quarter of the chunk that it contracts (k = (KC/4)*wave ..): nothing
  // staged is shared between wavefronts, so the chunk loop needs no barrier (one barrier per chunk cost 1.3 us of
  // the 34 us of the three-layer benchmark MLP).
  constexpr int A_QU = A_UPR / 4, B_QU = B_UPR / 4;  // units per row inside a quarter
  const int a_row0 = lane / A_QU, a_k = (KC / 4) * wave + (lane % A_QU) * AV;  // unit i sits in row a_row0 + i*(64/A_QU)
  const int b_row0 = lane / B_QU, b_k = (KC / 4) * wave + (lane % B_QU) * 4;
  static_assert(WAVE / A_QU == WG_THREADS / A_UPR && WAVE / B_QU == WG_THREADS / B_UPR, "row step of unit i");
  // load cursor: which chunk of which tile the next global loads fetch; row offsets are
  // recomputed only when the tile changes
  int ljob = vwg, lck = 0;
  // Per-lane BYTE offsets from the operands' base pointers, 32 bits (the host checks that both operands are
  // smaller than 4 GiB): a load is then "uniform 64-bit base + 32-bit lane offset" and costs no address arithmetic
  // on the vector ALU, which on this chip does not work while the matrix core does.
  unsigned aoff[A_LOADS], boff[B_LOADS];
  const char* Abase = reinterpret_cast<const char*>(A);
  const char* Wbase = reinterpret_cast<const char*>(Wl);
  auto point = [&]() {
    if (ljob >= njobs) return;
    // Column tiles vary fastest, so the workgroups of one XCD (ids equal modulo 8) share few weight rows.
    const int ct = ljob % tiles_m, rt = ljob / tiles_m;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++)
      aoff[i] = ((unsigned)min(rt * 16 + a_row0 + i * (WG_THREADS / A_UPR), batch - 1) * (unsigned)K + (unsigned)a_k) *
                (unsigned)sizeof(TA);
#pragma unroll
    for (int i = 0; i < B_LOADS; i++)
      boff[i] = ((unsigned)min(ct * 16 + b_row0 + i * (WG_THREADS / B_UPR), M - 1) * (unsigned)K + (unsigned)b_k) * 4u;
  };
  point();
  auto load_next = [&](Regs& r) {
    if (ljob >= njobs) return;
    const int k0 = lck * KC;
    if (k0 + KC <= K) {  // whole chunk inside the reduction: no per-lane checks (uniform branch)
      const char* Ak = Abase + (size_t)k0 * sizeof(TA);  // uniform
      const char* Wk = Wbase + (size_t)k0 * 4;
#pragma unroll
      for (int i = 0; i < A_LOADS; i++) r.a[i] = load_vec<TA, AV>(reinterpret_cast<const TA*>(Ak + aoff[i]));
#pragma unroll
      for (int i = 0; i < B_LOADS; i++) r.b[i] = load_vec<float, 4>(reinterpret_cast<const float*>(Wk + boff[i]));
    } else {  // ragged last chunk: clamp the address, zero what lies past K
      const bool ain = k0 + a_k < K, bin = k0 + b_k < K;
      const unsigned ashift = ain ? (unsigned)k0 * (unsigned)sizeof(TA) : 0u - (unsigned)a_k * (unsigned)sizeof(TA);
      const unsigned bshift = bin ? (unsigned)k0 * 4u : 0u - (unsigned)b_k * 4u;
#pragma unroll
      for (int i = 0; i < A_LOADS; i++) {
        r.a[i] = load_vec<TA, AV>(reinterpret_cast<const TA*>(Abase + (aoff[i] + ashift)));
#pragma unroll
        for (int e = 0; e < AV; e++) r.a[i].e[e] = ain ? r.a[i].e[e] : (TA)0;
      }
#pragma unroll
      for (int i = 0; i < B_LOADS; i++) {
        r.b[i] = load_vec<float, 4>(reinterpret_cast<const float*>(Wbase + (boff[i] + bshift)));
#pragma unroll
        for (int e = 0; e < 4; e++) r.b[i].e[e] = bin ? r.b[i].e[e] : 0.0f;
      }
    }
    if (++lck == nck) { lck = 0; ljob += step; point(); }
  };
  auto stage = [&](const Regs& r, char* buf) {
    TA* As = reinterpret_cast<TA*>(buf) + a_row0 * RSA + a_k;
    float* Bs = reinterpret_cast<float*>(buf + 16 * MLP_RS_D * 8) + b_row0 * MLP_RS_F + b_k;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      if constexpr (A64) {
        dbl2 t = {r.a[i].e[0], r.a[i].e[1]};
        *reinterpret_cast<dbl2*>(As + i * (WG_THREADS / A_UPR) * RSA) = t;
      } else {
        f4 t = {r.a[i].e[0], r.a[i].e[1], r.a[i].e[2], r.a[i].e[3]};
        *reinterpret_cast<f4*>(As + i * (WG_THREADS / A_UPR) * RSA) = t;
      }
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      f4 t = {r.b[i].e[0], r.b[i].e[1], r.b[i].e[2], r.b[i].e[3]};
      *reinterpret_cast<f4*>(Bs + i * (WG_THREADS / B_UPR) * MLP_RS_F) = t;
    }
  };

  Regs ring[NR];
#pragma unroll
  for (int i = 0; i < NR; i++) load_next(ring[i]);

  // Chunk t of the stream sits in ring[t % NR] until it is staged into LDS buffer t % 2.
  // Iteration t stages chunk t+1 (LDS writes and the next global loads are only issued
  // here) and then contracts chunk t, so both overlap the MFMAs; no barrier inside a tile.
  const int my_jobs = (njobs > vwg) ? (njobs - vwg + step - 1) / step : 0;
  const int total = my_jobs * nck;  // chunks in this workgroup's stream
  int job = vwg, ck = 0;
  d4 acc = d4_zero();
  double bz = (FC && job < njobs) ? (double)bias[min((job % tiles_m) * 16 + r16, M - 1)] : 0.0;
  if (total > 0) {
    stage(ring[0], smem);
    load_next(ring[0]);
  }
  __syncthreads();
  for (int t0 = 0; t0 < total; t0 += NR) {
#pragma unroll
    for (int i = 0; i < NR; i++) {
      const int t = t0 + i;
      if (t < total) {  // uniform over the workgroup
        char* buf = smem + (i & 1) * MLP_BUF_BYTES;
        // this wavefront's quarter of the chunk: k = (KC/4)*wave + 16*j + 4*q + e.  Its LDS reads are issued first,
        // the staging of the next chunk (LDS writes to the other buffer, the next global loads) runs while they are
        // in flight, the MFMAs come last: one LDS latency per chunk is hidden instead of two being paid.
        const TA* As = reinterpret_cast<const TA*>(buf) + r16 * RSA + (KC / 4) * wave + 4 * q;
        const float* Bs = reinterpret_cast<const float*>(buf + 16 * MLP_RS_D * 8) + r16 * MLP_RS_F + (KC / 4) * wave + 4 * q;
        // (a ragged tail was staged as zeros, so every step can run unconditionally)
        Vec<TA, 4> av[KC / 64];
        Vec<float, 4> bv[KC / 64];
#pragma unroll
        for (int j = 0; j < KC / 64; j++) {
          if constexpr (A64) {  // rows are 16-byte, not 32-byte, aligned: two 16-byte reads
            const Vec<TA, 2> lo = load_vec<TA, 2>(As + 16 * j), hi = load_vec<TA, 2>(As + 16 * j + 2);
            av[j].e[0] = lo.e[0]; av[j].e[1] = lo.e[1]; av[j].e[2] = hi.e[0]; av[j].e[3] = hi.e[1];
          } else {
            av[j] = load_vec<TA, 4>(As + 16 * j);
          }
          bv[j] = load_vec<float, 4>(Bs + 16 * j);
        }
        if (t + 1 < total) {
          stage(ring[(i + 1) % NR], smem + ((i + 1) & 1) * MLP_BUF_BYTES);
          load_next(ring[(i + 1) % NR]);
        }
#pragma unroll
        for (int j = 0; j < KC / 64; j++)
#pragma unroll
          for (int e = 0; e < 4; e++) acc = mfma_f64((double)av[j].e[e], (double)bv[j].e[e], acc);
        const bool last = (++ck == nck);
        d4* part = part_base + parity * (WAVES_PER_WG * WAVE);
        if (last) part[wave * WAVE + lane] = acc;
        if (last) __syncthreads();
        if (last) {
          // combine the four partial tiles in a fixed order, bias first (the listing's
          // first statement); wavefront w finishes rows 4w+q of the tile
          const int v = wave;
          double x = bz;
          x += part[0 * WAVE + lane][v];
          x += part[1 * WAVE + lane][v];
          x += part[2 * WAVE + lane][v];
          x += part[3 * WAVE + lane][v];
          if (FC) x = relu64(x);
          const int ct = job % tiles_m, rt = job / tiles_m;
          const int row = rt * 16 + d_row(q, v), col = ct * 16 + r16;
          if (row < batch && col < M) {
            const int64_t o = (int64_t)row * M + col;
            if (O) O[o] = (float)x;
            if (act) act_store(act + o, x);
          }
          ck = 0;
          parity ^= 1;
          job += step;
          acc = d4_zero();
          if (FC && job < njobs) bz = (double)bias[min((job % tiles_m) * 16 + r16, M - 1)];
        }
      }
    }
  }
  // the second team of a workgroup passes as many tile-end barriers as the first (it never has more tiles)
  for (int extra = my_jobs; extra < team0_jobs_if_team1; extra++) __syncthreads();
  __syncthreads();  // the LDS stage is reused by the next layer
}

// Teams (4 wavefronts that own a tile together) per workgroup.  Two workgroups of one team each per compute unit
// hold the same wavefronts, but the one dispatched second starts ~1 us later and finishes its first-layer tile 1.7 us
// after the other, and every workgroup of the grid waits for it at the barrier; two teams in one workgroup start
// together (and halve the barrier's participants): 33.1 -> 29.8 us for the three-layer benchmark MLP.
constexpr int MLP_TEAMS = 2;
__global__ __launch_bounds__(MLP_TEAMS * WG_THREADS, 2 / MLP_TEAMS) void mlp_fused_kernel(MlpArgs p) {
  extern __shared__ __attribute__((aligned(32))) char smem_all[];
  // team t of workgroup w is team t * gridDim + w of the grid: the first teams take the first tiles, as the first
  // workgroups of a two-per-unit launch would
  const int team = __builtin_amdgcn_readfirstlane(threadIdx.x / WG_THREADS);
  char* smem = smem_all + team * MLP_LDS_BYTES;
  const int vwg = team * (int)gridDim.x + (int)blockIdx.x, vstep = MLP_TEAMS * (int)gridDim.x;
  if (blockIdx.x == 0 && threadIdx.x == 0 && p.n_layers > 1) {
    const unsigned ngroups = (gridDim.x + MLP_FANIN - 1) / MLP_FANIN;
    for (int l = 0; l + 1 < p.n_layers; l++) {
      unsigned* bar = p.sync + MLP_SYNC_WORDS + l * MLP_BAR_WORDS;
      __hip_atomic_store(bar, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      for (unsigned g = 0; g < ngroups; g++) {
        __hip_atomic_store(bar + 16 + 16 * g, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // release words too: a graph replay carries the same token, so last time's would still match
        __hip_atomic_store(bar + 16 + 16 * MLP_GROUPS + 16 * g, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    __hip_atomic_store(p.sync + MLP_SYNC_EXIT, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p.sync + MLP_SYNC_ERROR, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p.sync + MLP_SYNC_TOKEN), p.token, __ATOMIC_RELEASE,
                       __HIP_MEMORY_SCOPE_AGENT);
  }
  for (int l = 0; l < p.n_layers; l++) {
    const int K = p.dims[l], M = p.dims[l + 1];
    double* act = (l + 1 < p.n_layers) ? p.act[l] : nullptr;
    int t0jobs = -1;
    if (team > 0) {
      const int njobs = ((p.batch + 15) / 16) * ((M + 15) / 16), b = (int)blockIdx.x;
      t0jobs = njobs > b ? (njobs - b + vstep - 1) / vstep : 0;
    }
    if (l == 0)
      mlp_layer<float>(p.I, p.W[0], p.bias[0], p.O[0], act, p.batch, K, M, smem, vwg, vstep, t0jobs);
    else
      mlp_layer<double>(p.act[l - 1], p.W[l], p.bias[l], p.O[l], act, p.batch, K, M, smem, vwg, vstep, t0jobs);
    if (l + 1 < p.n_layers) mlp_grid_barrier(p.sync, l, p.token, gridDim.x, p.spin_limit);
  }
  // The last workgroup out withdraws the token.  A replay of a captured HIP graph launches this
  // kernel again with the SAME token; with the token withdrawn, the other workgroups again wait
  // until workgroup 0 has zeroed the counters before they count themselves in.
  if (p.n_layers > 1 && threadIdx.x == 0) {
    const unsigned old = __hip_atomic_fetch_add(p.sync + MLP_SYNC_EXIT, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == gridDim.x - 1)
      __hip_atomic_store(reinterpret_cast<unsigned long long*>(p.sync + MLP_SYNC_TOKEN), 0ull, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
  }
}

// One contraction C[N][M] = sum_k A[N][k] * Bm[M][k] with the layer body above: 16 x 16 output tiles dealt to
// persistent workgroups whose four wavefronts split every chunk of the reduction.  For one matrix pair (no batch
// stride) with a long reduction and too few 64 x 64 blocks to fill the chip.
__global__ __launch_bounds__(WG_THREADS, 2) void gemm_nt_splitk_kernel(GemmArgs p) {
  extern __shared__ __attribute__((aligned(32))) char smem[];
  mlp_layer<float, false>(static_cast<const float*>(p.A), p.Bm, nullptr, p.C, nullptr, p.N, p.K, p.M, smem,
                          (int)blockIdx.x, (int)gridDim.x, -1);
}

}  // namespace tc355
