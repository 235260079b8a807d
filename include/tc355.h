/*
 * tc355.h -- C ABI of libtc355: evaluation of tensor comprehensions on one
 * AMD MI355X (gfx950).
 *
 * A tensor comprehension (arXiv 1802.04730, Section 3) is an index-notation
 * statement: every output element is a sum, over the indices that appear only
 * on the right-hand side, of a product of tensor accesses, optionally followed
 * by a pointwise epilogue.  This library evaluates six fixed comprehensions.
 *
 * Conventions common to every entry point
 *  - Every tensor pointer is a DEVICE pointer to a dense row-major array (last
 *    index fastest, Section 5 "row-major arrays"), fp32 storage, base address
 *    a multiple of 16 bytes.  The caller owns all tensors, outputs included
 *    (Section 3.1: memory management is left to the calling framework), and
 *    keeps them alive until the stream has run the work.
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *    the default stream).  Calls are asynchronous: the library never
 *    synchronises, allocates or frees device memory.
 *  - Outputs need not be zeroed: a "+=!" reduction starts from 0 (Section 3).
 *  - Outputs must not overlap inputs.  Equal base pointers are rejected with
 *    TC_ERR_ALIAS; other overlap is undefined.
 *  - Arithmetic: inputs are widened exactly to fp64, products and sums are
 *    taken in fp64 (fp64 matrix-core instructions), and each declared output
 *    is rounded once to fp32.  Values handed from one stage of a chain to the
 *    next stay in fp64.  The exceptions, see tc_group_conv and tc_tbmm: some
 *    16- and 32-channel 3 x 3 grouped convolutions and the transposed matmul
 *    with 128 rows sum exactly in integers over operands quantised to 2^-32
 *    of their block maximum.
 *  - Validation precedes any launch: on a non-zero status nothing was written.
 *    A batch extent of 0 returns TC_OK without launching.
 *  - Thread safety: the only mutable global state is a per-process cache of
 *    device properties and an atomic call counter; concurrent calls from
 *    several host threads are allowed.
 *  - No environment variable is read.  The few switches (arithmetic of the
 *    int8 paths, choice of MLP kernel, spin limit of its waits) are options of
 *    the calling host thread: tc355_set_option below.
 */
#ifndef TC355_H
#define TC355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TC_OK = 0,
  TC_ERR_NULL = 1,      /* a required pointer is NULL                          */
  TC_ERR_SHAPE = 2,     /* an extent is <= 0, or an inferred extent is <= 0    */
  TC_ERR_ALIAS = 3,     /* an output base pointer equals an input base pointer */
  TC_ERR_ALIGN = 4,     /* a base pointer is not 16-byte aligned               */
  TC_ERR_WORKSPACE = 5, /* workspace missing, misaligned or too small          */
  TC_ERR_LAUNCH = 6,    /* the HIP runtime refused the launch                  */
  TC_ERR_UNSUPPORTED = 7, /* extents beyond what the kernels index (>= 2^31 elements per tensor) */
  TC_ERR_SCRATCH_LIMIT = 8 /* tc_mlp_fcrelu_static: the call needs more than TC_MLP_STATIC_SCRATCH_BYTES */
} tc_status;

/* Human-readable name of a status; static storage, never freed. */
const char *tc_status_string(tc_status s);

/* Library version: major*10000 + minor*100 + patch. */
int tc355_version(void);

/*
 * Options of the CALLING HOST THREAD (thread-local: they affect the calls this
 * thread makes afterwards and race with nothing).  Meant for tests, benchmarks
 * and for callers that know their data; the defaults are safe for any input.
 *   TC_OPT_INT8            arithmetic of the shapes that have an int8 matrix-core
 *                          path (see tc_group_conv, tc_tbmm, tc_sconv2d):
 *       TC_INT8_AUTO       (default) sliced int8 arithmetic; blocks whose operands
 *                          are heavy-tailed get 13 instead of 10 digit products
 *       TC_INT8_OFF        the fp64 path for every shape
 *       TC_INT8_TEN        10 digit products for every block (fastest; accuracy
 *                          then depends on the data, see tc_group_conv)
 *       TC_INT8_THIRTEEN   13 digit products for every block
 *   TC_OPT_MLP_KERNEL      TC_MLP_AUTO (default), TC_MLP_ROWS, TC_MLP_TILES (one
 *                          persistent kernel of either kind where it applies),
 *                          TC_MLP_PER_LAYER (one launch per layer)
 *   TC_OPT_MLP_SPIN_LIMIT  polls that a wait inside a fused MLP kernel may make before
 *                          it gives up (default 4000000; >= 0).  0: every wait for
 *                          another workgroup's results gives up without looking, so
 *                          the call is certain to end with the error word raised
 *                          (what the tests of that path use)
 * tc355_set_option returns TC_ERR_SHAPE for an unknown key or a value out of
 * range.  tc355_get_option returns the current value (-1 for an unknown key).
 */
typedef enum { TC_OPT_INT8 = 0, TC_OPT_MLP_KERNEL = 1, TC_OPT_MLP_SPIN_LIMIT = 2 } tc_option;
enum { TC_INT8_AUTO = 0, TC_INT8_OFF = 1, TC_INT8_TEN = 2, TC_INT8_THIRTEEN = 3 };
enum { TC_MLP_AUTO = 0, TC_MLP_ROWS = 1, TC_MLP_TILES = 2, TC_MLP_PER_LAYER = 3 };
tc_status tc355_set_option(tc_option key, int64_t value);
int64_t tc355_get_option(tc_option key);

/*
 * Which kernel family the calling thread's most recent entry-point call chose,
 * as a static string "op:family" (for example "tbmm:lds", "tbmm:i8",
 * "mlp:rows", "gconv:i8", "gconv:i8_taps", "gconv:band", "sconv:i8", "sconv:tile",
 * "lut:sum"; ""
 * before the first call).  A debugging and testing aid: tests pick the tolerance of the
 * arithmetic that actually ran instead of re-deriving the dispatch.
 */
const char *tc355_last_path(void);

/*
 * Transposed batched matmul (Section 7, "Transposed Batched Matrix
 * Multiplication", listing tbmm; index names as in the benchmark
 * configurations):
 *     Z(b,n,m) +=! X(b,n,k) * Y(b,m,k)
 * X: [B,N,K]   Y: [B,M,K]   Z: [B,N,M]  (all device, fp32).
 * The reduction index is the fastest index of both operands.  B = 1 gives the
 * transposed matmul of Section 7 (listing tmm).
 * Arithmetic: fp64 products and sums, one rounding to fp32 -- except for
 * N a multiple of 128 with K a multiple of 4 (at least 256), M a multiple
 * of 64 and at least 128 blocks of 128 x 64 outputs in all (the paper's (M,K,N) =
 * (128,4096,16384) is of this kind), which run on the int8 matrix core: in
 * every block of 128 reduction indices (the last one filled with zeros where
 * K is no multiple of 128) each row of X and of Y is scaled so that
 * its largest magnitude m maps to 0x7F7F7F7E, rounded to a 32-bit integer
 * (off by at most 2^-32 m) and cut into four signed 8-bit digits; the 13 digit
 * products of weight 256^2 and above (digit k of one operand times digit l
 * of the other with k + l >= 2) are summed exactly in int32, scaled back
 * and added over the blocks in fp64, and the sum is rounded to fp32 once.
 * Error bound: K * 2^-30.5 * max|X row block| * max|Y row block| absolute,
 * worst case (the rounding of the two operands; the dropped digit products
 * are 2^-7 of that); on max|gpu - ref| / (|ref| + 1e-3 max|ref|) below 2e-6
 * for uniform, Gaussian and log-normal (sigma 2 on both operands) data.
 * With option TC_OPT_INT8 = TC_INT8_TEN the diagonal k + l = 2 is dropped
 * (10 products, K * 2^-29.5: 3e-7 .. 9e-7 for uniform and Gaussian operands,
 * up to 1.2e-5 for log-normal magnitudes of sigma 2), with TC_INT8_OFF these
 * shapes take the fp64 path too.  A row of X (of Y) that holds Inf or NaN
 * gives NaN in all of that row's (column's) outputs.
 */
tc_status tc_tbmm(const float *X, const float *Y, float *Z, int64_t B,
                  int64_t N, int64_t M, int64_t K, void *hip_stream);

/*
 * tc_tbmm with an optional workspace (same comprehension, Section 7, listings
 * tbmm / tmm; same results to the stated accuracy).  The shape class that runs
 * on the int8 matrix core (see tc_tbmm) spends a third of its vector work on
 * slicing X into 8-bit digits again in every workgroup that reads it; with a
 * workspace X is sliced once, by a kernel of its own launched first on the
 * same stream, and the contraction reads the digits.
 *   workspace        device scratch of at least tc_tbmm_workspace_bytes(...)
 *                    bytes, 16-byte aligned, distinct from X, Y and Z; contents
 *                    on entry are irrelevant, contents on return unspecified;
 *                    calls that share a workspace must be ordered on one stream.
 *                    NULL, or fewer bytes than needed, is not an error: the call
 *                    then does exactly what tc_tbmm does.
 * tc_tbmm_workspace_bytes returns 0 for shapes that would not use a workspace
 * (and on bad input); for those tc_tbmm_ws ignores the argument.
 */
size_t tc_tbmm_workspace_bytes(int64_t B, int64_t N, int64_t M, int64_t K);
tc_status tc_tbmm_ws(const float *X, const float *Y, float *Z, int64_t B,
                     int64_t N, int64_t M, int64_t K, void *workspace,
                     size_t workspace_bytes, void *hip_stream);

/*
 * Chain of n_layers fully connected + bias + ReLU layers, evaluated by one
 * call (Section 3, listing fcrelu; appendix "Production Models", listings
 * MLP1 (n_layers = 1) and MLP3 (n_layers = 3)).  For layer l = 0..n_layers-1
 *     O_l(b,n)  = bias_l(n)
 *     O_l(b,n) += In_l(b,m) * W_l(n,m)
 *     O_l(b,n)  = fmaxf(O_l(b,n), 0)
 * with In_0 = I and In_{l+1} = O_l.
 *   I        device [batch, dims[0]]
 *   dims     HOST array of n_layers+1 extents: dims[0] input width,
 *            dims[l+1] width of layer l
 *   W        HOST array of n_layers device pointers, W[l]: [dims[l+1], dims[l]]
 *   bias     HOST array of n_layers device pointers, bias[l]: [dims[l+1]]
 *   O        HOST array of n_layers device pointers, O[l]: [batch, dims[l+1]];
 *            O[n_layers-1] is required, O[l] for earlier layers may be NULL
 *            (that intermediate is then not written as fp32 at all)
 *   workspace  device scratch of at least tc_mlp_fcrelu_workspace_bytes(...)
 *            bytes, 256-byte aligned.  Its head holds the counters of the
 *            device-wide synchronisation between layers; the rest carries
 *            the fp64 activations from one layer to the next.  Contents on
 *            entry are irrelevant (the kernel initialises what it needs);
 *            calls that share a workspace must be ordered on one stream.  May
 *            be NULL when the required size is 0 (n_layers == 1).  After the
 *            call has run, 32-bit word 33 of the workspace is 1 if a
 *            device-wide wait gave up (workgroups could not all be resident
 *            at once; outputs are then unspecified) and 0 otherwise.
 * When every reduction extent dims[l] is a multiple of 4 the whole chain runs
 * as one persistent kernel; otherwise one kernel per layer is launched.
 * The persistent kernel's workgroups wait for one another, so it wants the
 * device to itself while it runs: kernels running at the same time on other
 * streams delay it (two chains on two streams were measured at 2.6 times the
 * time per call of one after the other, with correct results), and if its
 * workgroups cannot all become resident its waits give up (the error word
 * above).  TC_OPT_MLP_KERNEL = TC_MLP_PER_LAYER has no such waits.
 * The host arrays are read before the call returns.  1 <= n_layers <= 8.
 * The clamp maps NaN and -0 to +0, like fmaxf(x, 0).
 */
tc_status tc_mlp_fcrelu(const float *I, int64_t batch, int32_t n_layers,
                        const int64_t *dims, const float *const *W,
                        const float *const *bias, float *const *O,
                        void *workspace, size_t workspace_bytes,
                        void *hip_stream);

/* Bytes of workspace tc_mlp_fcrelu needs for these extents (0 on bad input). */
size_t tc_mlp_fcrelu_workspace_bytes(int64_t batch, int32_t n_layers,
                                     const int64_t *dims);

/*
 * tc_mlp_fcrelu for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and same
 * results as tc_mlp_fcrelu, but the scratch (synchronisation words and fp64
 * activations) is a static device array inside the library instead of a
 * workspace argument.  The call allocates and frees nothing.
 *   - Limit: tc_mlp_fcrelu_workspace_bytes(batch, n_layers, dims) must not
 *     exceed TC_MLP_STATIC_SCRATCH_BYTES (8 MiB, enough for the benchmark's
 *     128 x 1024 -> 1024 -> 512 -> 256 chain four times over); beyond it the
 *     call returns TC_ERR_SCRATCH_LIMIT and launches nothing.
 *   - Every GPU the library runs on holds its own copy of the array until the
 *     process ends.  Its device address is looked up once per device, at the
 *     first call on that device (make that first call outside a capture).
 *   - All calls on one GPU share that GPU's array and it keeps the previous
 *     call's contents; the kernel initialises the words it needs, so nothing
 *     has to be cleared between calls.  Calls that overlap in time on one GPU
 *     (different streams, different host threads) race on it: order them.
 */
#define TC_MLP_STATIC_SCRATCH_BYTES (8u << 20)
tc_status tc_mlp_fcrelu_static(const float *I, int64_t batch, int32_t n_layers,
                               const int64_t *dims, const float *const *W,
                               const float *const *bias, float *const *O,
                               void *hip_stream);

/*
 * Grouped 2-D convolution, stride 1, no padding, plus per-output-channel bias
 * (Section 7, "Grouped Convolutions", listing gconv):
 *     O(n,g,o,h,w) +=! I(n,g,i,h+kh,w+kw) * W1(g,o,i,kh,kw)
 *     O(n,g,o,h,w)  =  O(n,g,o,h,w) + bias(g*F+o)
 * I: [N,G,C,H,W] (= NCHW with G*C channels)   W1: [G,F,C,KH,KW]
 * bias: [G*F] or NULL (no bias statement)      O: [N,G,F,H-KH+1,W-KW+1].
 * Output extents follow range inference (Section 3.1); H < KH or W < KW gives
 * TC_ERR_SHAPE.
 * Arithmetic: fp64 as everywhere, except for C = F = 16, KH = KW = 3 with
 * W = 58, H even and H - 2 a multiple of 8 (the benchmark's geometry) or with
 * H = W = 14 or 16 and N a multiple of 4 (and for C = F = 32, KH = KW = 3,
 * H = W = 7, N a multiple of 4), which run on
 * the int8 matrix core: every filter row and every band of 10 input rows
 * (for 14 x 14: every whole block of 16 input planes) is
 * scaled to 32-bit fixed point (the block's largest magnitude maps to
 * 0x7F7F7F7E, every element is held to 2^-32 of that magnitude), cut into
 * four signed 8-bit digits; digit products (digit k of a filter element
 * times digit l of an input element) are summed exactly in int32, the
 * result is recombined in fp64, the bias added, and rounded to fp32 once.
 * The 10 products with k + l >= 3 are always taken; the three with
 * k + l = 2 are worth up to K * 2^-29.5 * max|filter row| * max|band| over a
 * reduction of K terms, which is far below the outputs unless BOTH operands
 * are heavy-tailed (a few elements far above the rest in every band and
 * every filter row, so that the block maxima say little about the outputs).
 * The 14 x 14 and 7 x 7 geometries always take them (13 products).  The
 * width-58 geometry decides per thread (one band of one image with the 16
 * filter rows of its group): with S = (band maximum / smallest maximum among
 * the band's four column strips) * (largest ratio of maximum to mean
 * magnitude among the 16 filter rows), it takes the 10 products when
 * S <= 128 (Gaussian and ReLU-like data: S = 11 .. 22, Laplace up to 72) and
 * adds the three others in extra sweeps otherwise (log-normal, Student-t,
 * sparse outliers: S from 150 up), at about 40 % more time for such
 * a thread.  Either way the error against the float64 definition stays
 * below 5e-6 on the parity metric max|err| / (|ref| + 1e-3 max|ref|) for
 * all of these distributions (1e-6 for the benchmark's).
 * Option TC_OPT_INT8: TC_INT8_TEN never takes the diagonal (1.6e-5
 * measured with log-normal magnitudes of sigma 1.5 and 1), TC_INT8_THIRTEEN
 * always does, TC_INT8_OFF takes the fp64 path.  A band that holds Inf or NaN
 * gives NaN in all outputs that read the band.
 * Groups with F a multiple of 32 and C*KH*KW a multiple of 4 and at least 256
 * (G = 1 with such extents is the plain convolution of Section 3) run on the
 * int8 kernel of tc_sconv2d with stride 1, one group after the other in one
 * launch: its arithmetic (blocks of 128 taps, a scale per filter and per
 * output pixel in every block, 13 digit products; TC_INT8_TEN: 10), its
 * limits and its Inf/NaN behaviour are described there.
 */
tc_status tc_group_conv(const float *I, const float *W1, const float *bias,
                        float *O, int64_t N, int64_t G, int64_t C, int64_t F,
                        int64_t H, int64_t W, int64_t KH, int64_t KW,
                        void *hip_stream);

/*
 * Output extents of tc_group_conv by range inference (Section 3.1: the output
 * index h keeps h+kh inside the input for every kh, hence H-KH+1 values).
 * Host only; touches no GPU.  OH, OW: host pointers.
 */
tc_status tc_group_conv_infer(int64_t H, int64_t W, int64_t KH, int64_t KW,
                              int64_t *OH, int64_t *OW);

/*
 * Kronecker-factored linear layer (benchmark configuration 5; semantics of
 * Section 3):
 *     Y(b,i,j) +=! W1(i,k) * W2(j,l) * X(b,k,l)
 * W1: [I,K]   W2: [J,L]   X: [B,K,L]   Y: [B,I,J].
 * Evaluated as two chained contractions, T(b,i,l) = sum_k W1(i,k) X(b,k,l)
 * then Y(b,i,j) = sum_l T(b,i,l) W2(j,l); T stays on chip in fp64.
 */
tc_status tc_kron(const float *W1, const float *W2, const float *X, float *Y,
                  int64_t B, int64_t I, int64_t K, int64_t J, int64_t L,
                  void *hip_stream);

/*
 * Strided 2-D convolution, no padding, per-output-channel bias (Section 3,
 * listing sconv2d):
 *     O(n,f,h,w)  = B(f)
 *     O(n,f,h,w) += I(n,c, sh*h + kh, sw*w + kw) * W(f,c,kh,kw)
 * I: [N,C,H,W]   Wt: [F,C,KH,KW]   bias: [F] or NULL (the first statement
 * then assigns 0)   O: [N,F,OH,OW] with OH = (H-KH)/sh + 1, OW = (W-KW)/sw + 1
 * (integer division; see tc_sconv2d_infer).  sh, sw >= 1; sh = sw = 1 is the
 * plain convolution.  H < KH or W < KW gives TC_ERR_SHAPE.  Arithmetic: fp64
 * products and sums, one rounding per output -- except for F a multiple of 32
 * with C*KH*KW a multiple of 4, at least 256 and at most about 17,000 (I below
 * 2^30 elements, O below 2^31), which run on the int8 matrix core by the scheme of
 * tc_tbmm: the reduction index (c,kh,kw), in W's order, is cut into blocks of
 * 128 (the last one filled with zeros); in every block each filter and each
 * output pixel's taps are scaled to 0x7F7F7F7E by their own largest magnitude,
 * rounded to a 32-bit integer and cut into four signed 8-bit digits; the 13
 * digit products of weight 256^2 and above are summed exactly in int32, scaled
 * back and added over the blocks in fp64; bias added in fp64, one rounding to
 * fp32.  Error bound and measured errors as for tc_tbmm (C*KH*KW for K);
 * TC_OPT_INT8 = TC_INT8_TEN drops the lowest diagonal (10 products),
 * TC_INT8_OFF keeps the fp64 kernel.  On the int8 path a NaN or an Inf among
 * an output's own taps, or anywhere in its filter, gives NaN (the exact sum
 * would give an Inf where every infinite product has the same sign).
 */
tc_status tc_sconv2d(const float *I, const float *Wt, const float *bias,
                     float *O, int64_t N, int64_t C, int64_t F, int64_t H,
                     int64_t W, int64_t KH, int64_t KW, int64_t sh, int64_t sw,
                     void *hip_stream);

/*
 * Output extents of tc_sconv2d by range inference (Section 3.1): h takes every
 * value for which sh*h + kh is a row of I for all kh < KH, i.e. sh*h <= H-KH.
 * Host only; touches no GPU.  OH, OW: host pointers.
 */
tc_status tc_sconv2d_infer(int64_t H, int64_t W, int64_t KH, int64_t KW,
                           int64_t sh, int64_t sw, int64_t *OH, int64_t *OW);

/*
 * Lookup-table sums, n_tables of them in one launch (Section 7, production
 * model; appendix listing 2LUT, which is n_tables = 2; its single-table form
 * 1LUT is n_tables = 1).  For every table t:
 *     O_t(i,j) +=! LUT_t(Idx_t(i,k), j)        i < B, j < D, k < L[t]
 *   LUT   HOST array of n_tables device pointers, LUT[t]: [E[t], D] fp32
 *   Idx   HOST array of n_tables device pointers, Idx[t]: [B, L[t]] int32
 *   O     HOST array of n_tables device pointers, O[t]: [B, D] fp32
 *   E, L  HOST arrays of n_tables extents; D and B are common to all tables
 * 1 <= n_tables <= 8; E[t] <= 2^31.  The host arrays are read before the call
 * returns.  An index that occurs several times in a row of Idx counts as
 * often.  The comprehension gives no meaning to an index outside [0, E[t]):
 * the kernel reads nothing for it and writes NaN to the whole output row i of
 * that table (indices live on the device, so the host cannot reject them).
 * Arithmetic: the gathered values are summed in fp64 and rounded to fp32 once.
 */
tc_status tc_lut(int32_t n_tables, const float *const *LUT,
                 const int32_t *const *Idx, float *const *O, const int64_t *E,
                 const int64_t *L, int64_t D, int64_t B, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TC355_H */
