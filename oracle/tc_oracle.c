/*
 * tc_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, float64 CPU evaluator of the tensor comprehensions the GPU
 * library implements (transposed batched matmul, fcrelu chain, grouped
 * convolution, Kronecker layer, strided convolution, lookup-table sum).  Every function is the loop nest that the paper's
 * Section 3 ("Tensor Comprehensions") gives as the meaning of a
 * comprehension: one "parallel for" per left-hand-side index, one
 * "reduction for" per index that appears on the right only, the body being
 * the statement itself.  A "+=!" reduction starts from the neutral element 0
 * (Section 3, initialising reductions); a "=" statement followed by "+="
 * accumulates onto the assigned value (Section 3, fcrelu listing).
 *
 * Inputs are the caller's fp32 values; they are widened exactly to double,
 * every product and every sum is taken in double, and the result is left in
 * double.  No blocking, no reordering, no fusion beyond what the listings
 * state.  The only concession to run time is an OpenMP "parallel for" on the
 * outermost *parallel* (left-hand-side) index, which the semantics allow
 * (Section 3: evaluation order of iteration points does not affect the
 * output); reductions are never split, so the result does not depend on the
 * number of threads.
 *
 * This file shares nothing with the HIP path: no header, no helper, no table.
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
 * call it.
 *
 * Pins (tests/test_oracle_*.py): brute-force Python loops on tiny shapes,
 * numpy/torch float64 library routines (einsum, matmul, conv2d with groups,
 * kron), closed forms (identity operands, delta filters, all-zero weights),
 * invariants (ReLU >= 0, G=1 equals ordinary convolution, the Kronecker
 * vec identities) and planted-mistake checks.  The paper prints no numeric
 * input->output example, so there is no printed value to match.
 *
 * The strided convolution is pinned against torch's conv2d with a stride, the
 * stride-1 case, subsampling of the stride-1 result, delta filters and loops;
 * the lookup-table sum against a one-hot matrix product, plain fancy indexing,
 * a closed form on an affine table and loops; the inferred extents of the
 * strided convolution against a count over the quantified definition.
 *
 * Return value of every evaluator: 0 on success, 1 null pointer, 2 bad shape
 * (tc_oracle_lut: 3 if an index lies outside the table).
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of OpenMP threads used for the outermost parallel index (>=1). */
void tc_oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int tc_oracle_get_threads(void) {
#ifdef _OPENMP
  return g_threads;
#else
  return 1;
#endif
}

int tc_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_num_procs();
#else
  return 1;
#endif
}

/*
 * Transposed batched matmul (Section 7, "Transposed Batched Matrix
 * Multiplication", listing tbmm), with the index names of the benchmark
 * configuration:   Z(b,n,m) +=! X(b,n,k) * Y(b,m,k)
 * X is [B,N,K], Y is [B,M,K], Z is [B,N,M]; all dense row-major.
 * (The paper's listing names the same three roles n,k,m -- the reduction is
 * over the last index of both operands either way.)
 */
int tc_oracle_tbmm(const float *X, const float *Y, double *Z, int64_t B,
                   int64_t N, int64_t M, int64_t K) {
  if (!X || !Y || !Z) return 1;
  if (B < 0 || N <= 0 || M <= 0 || K <= 0) return 2;
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t b = 0; b < B; b++)
    for (int64_t n = 0; n < N; n++)
      for (int64_t m = 0; m < M; m++) {
        double z = 0.0; /* "+=!" : neutral element of + */
        for (int64_t k = 0; k < K; k++)
          z += (double)X[(b * N + n) * K + k] * (double)Y[(b * M + m) * K + k];
        Z[(b * N + n) * M + m] = z;
      }
  return 0;
}

/*
 * Chain of fully connected + bias + ReLU layers (Section 3, listing fcrelu;
 * appendix "Production Models", listings MLP1 and MLP3).  For layer l:
 *     O_l(b,n)  = bias_l(n)
 *     O_l(b,n) += In_l(b,m) * W_l(n,m)
 *     O_l(b,n)  = fmaxf(O_l(b,n), 0)
 * with In_0 = I and In_{l+1} = O_l.  dims[0] is the input width, dims[l+1]
 * the width of layer l; W[l] is [dims[l+1], dims[l]], bias[l] is
 * [dims[l+1]], O[l] is [batch, dims[l+1]] in double.  The chain is carried
 * in double from layer to layer (no rounding of O_l to float in between);
 * round_intermediates != 0 selects the diagnostic variant that rounds each
 * O_l to float before it feeds the next layer.
 * The clamp is written x > 0 ? x : 0, which sends NaN and -0 to +0.
 */
int tc_oracle_mlp_fcrelu(const float *I, int64_t batch, int32_t n_layers,
                         const int64_t *dims, const float *const *W,
                         const float *const *bias, double *const *O,
                         int32_t round_intermediates) {
  if (!I || !dims || !W || !bias || !O) return 1;
  if (batch < 0 || n_layers <= 0) return 2;
  for (int32_t l = 0; l <= n_layers; l++)
    if (dims[l] <= 0) return 2;
  for (int32_t l = 0; l < n_layers; l++)
    if (!W[l] || !bias[l] || !O[l]) return 1;

  for (int32_t l = 0; l < n_layers; l++) {
    const int64_t Min = dims[l], Nout = dims[l + 1];
    const float *Wl = W[l];
    const float *bl = bias[l];
    const double *prev = l ? O[l - 1] : NULL;
    double *out = O[l];
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t b = 0; b < batch; b++)
      for (int64_t n = 0; n < Nout; n++) {
        double o = (double)bl[n];
        for (int64_t m = 0; m < Min; m++) {
          double in;
          if (l == 0)
            in = (double)I[b * Min + m];
          else if (round_intermediates)
            in = (double)(float)prev[b * Min + m];
          else
            in = prev[b * Min + m];
          o += in * (double)Wl[n * Min + m];
        }
        out[b * Nout + n] = o > 0.0 ? o : 0.0;
      }
  }
  return 0;
}

/*
 * Output extents of the convolution by range inference (Section 3.1 "Range
 * Inference": the reduction indices take the full filter extent first, then
 * the output index h must keep h+kh in bounds for every kh, which leaves
 * H-KH+1 values).  Returns 2 if either extent would be empty.
 */
int tc_oracle_group_conv_infer(int64_t H, int64_t W, int64_t KH, int64_t KW,
                               int64_t *OH, int64_t *OW) {
  if (!OH || !OW) return 1;
  if (H <= 0 || W <= 0 || KH <= 0 || KW <= 0) return 2;
  if (H - KH + 1 <= 0 || W - KW + 1 <= 0) return 2;
  *OH = H - KH + 1;
  *OW = W - KW + 1;
  return 0;
}

/*
 * Grouped convolution, stride 1, no padding (Section 7, "Grouped
 * Convolutions", listing gconv):
 *     O(n,g,o,h,w) +=! I(n,g,i,h+kh,w+kw) * W1(g,o,i,kh,kw)
 *     O(n,g,o,h,w)  =  O(n,g,o,h,w) + B(g*F+o)
 * I is [N,G,C,H,W], W1 is [G,F,C,KH,KW], B is [G*F] (may be NULL: no bias
 * statement), O is [N,G,F,H-KH+1,W-KW+1].  The bias index is the output
 * channel g*F+o, as the generated kernel in the appendix reads it.
 */
int tc_oracle_group_conv(const float *I, const float *W1, const float *Bv,
                         double *O, int64_t N, int64_t G, int64_t C, int64_t F,
                         int64_t H, int64_t W, int64_t KH, int64_t KW) {
  int64_t OH, OW;
  if (!I || !W1 || !O) return 1;
  if (N < 0 || G <= 0 || C <= 0 || F <= 0) return 2;
  if (tc_oracle_group_conv_infer(H, W, KH, KW, &OH, &OW)) return 2;
#pragma omp parallel for num_threads(g_threads) schedule(static) collapse(2)
  for (int64_t n = 0; n < N; n++)
    for (int64_t g = 0; g < G; g++)
      for (int64_t o = 0; o < F; o++)
        for (int64_t h = 0; h < OH; h++)
          for (int64_t w = 0; w < OW; w++) {
            double s = 0.0;
            for (int64_t i = 0; i < C; i++)
              for (int64_t kh = 0; kh < KH; kh++)
                for (int64_t kw = 0; kw < KW; kw++)
                  s += (double)I[(((n * G + g) * C + i) * H + (h + kh)) * W +
                                 (w + kw)] *
                       (double)W1[(((g * F + o) * C + i) * KH + kh) * KW + kw];
            if (Bv) s = s + (double)Bv[g * F + o];
            O[(((n * G + g) * F + o) * OH + h) * OW + w] = s;
          }
  return 0;
}

/*
 * Kronecker-factored linear layer, as ONE five-index comprehension (benchmark
 * configuration 5; the paper has no listing for it, the semantics are those
 * of Section 3):
 *     Y(b,i,j) +=! W1(i,k) * W2(j,l) * X(b,k,l)
 * W1 is [I,K], W2 is [J,L], X is [B,K,L], Y is [B,I,J].  The product of the
 * three accesses is taken left to right in double.  The two-stage
 * factorisation is the GPU's method and is deliberately not used here.
 */
int tc_oracle_kron(const float *W1, const float *W2, const float *X, double *Y,
                   int64_t B, int64_t I, int64_t K, int64_t J, int64_t L) {
  if (!W1 || !W2 || !X || !Y) return 1;
  if (B < 0 || I <= 0 || K <= 0 || J <= 0 || L <= 0) return 2;
#pragma omp parallel for num_threads(g_threads) schedule(static) collapse(2)
  for (int64_t b = 0; b < B; b++)
    for (int64_t i = 0; i < I; i++)
      for (int64_t j = 0; j < J; j++) {
        double y = 0.0;
        for (int64_t k = 0; k < K; k++)
          for (int64_t l = 0; l < L; l++)
            y += (double)W1[i * K + k] * (double)W2[j * L + l] *
                 (double)X[(b * K + k) * L + l];
        Y[(b * I + i) * J + j] = y;
      }
  return 0;
}

/*
 * Output extents of the strided convolution by range inference (Section 3.1
 * "Range Inference"): kh and kw take the full filter extent from W; the
 * output index h may take every value for which sh*h + kh stays inside
 * [0, H) for ALL kh < KH, i.e. sh*h <= H - KH: floor((H-KH)/sh) + 1 values
 * (likewise for w).  Returns 2 if an extent, a stride or a range is empty.
 */
int tc_oracle_sconv2d_infer(int64_t H, int64_t W, int64_t KH, int64_t KW,
                            int64_t sh, int64_t sw, int64_t *OH, int64_t *OW) {
  if (!OH || !OW) return 1;
  if (H <= 0 || W <= 0 || KH <= 0 || KW <= 0 || sh <= 0 || sw <= 0) return 2;
  if (H < KH || W < KW) return 2;
  *OH = (H - KH) / sh + 1;
  *OW = (W - KW) / sw + 1;
  return 0;
}

/*
 * Strided convolution (Section 3, listing sconv2d):
 *     O(n,f,h,w)  = B(f)
 *     O(n,f,h,w) += I(n,c, sh*h + kh, sw*w + kw) * W(f,c,kh,kw)
 * I is [N,C,H,W], Wt is [F,C,KH,KW], Bv is [F] (may be NULL: the first
 * statement then assigns 0), O is [N,F,OH,OW] with the inferred extents.
 * The bias is assigned first and the products accumulate onto it, in the
 * order of the listing.
 */
int tc_oracle_sconv2d(const float *I, const float *Wt, const float *Bv,
                      double *O, int64_t N, int64_t C, int64_t F, int64_t H,
                      int64_t W, int64_t KH, int64_t KW, int64_t sh,
                      int64_t sw) {
  int64_t OH, OW;
  if (!I || !Wt || !O) return 1;
  if (N < 0 || C <= 0 || F <= 0) return 2;
  if (tc_oracle_sconv2d_infer(H, W, KH, KW, sh, sw, &OH, &OW)) return 2;
#pragma omp parallel for num_threads(g_threads) schedule(static) collapse(2)
  for (int64_t n = 0; n < N; n++)
    for (int64_t f = 0; f < F; f++)
      for (int64_t h = 0; h < OH; h++)
        for (int64_t w = 0; w < OW; w++) {
          double o = Bv ? (double)Bv[f] : 0.0;
          for (int64_t c = 0; c < C; c++)
            for (int64_t kh = 0; kh < KH; kh++)
              for (int64_t kw = 0; kw < KW; kw++)
                o += (double)I[((n * C + c) * H + (sh * h + kh)) * W +
                               (sw * w + kw)] *
                     (double)Wt[((f * C + c) * KH + kh) * KW + kw];
          O[((n * F + f) * OH + h) * OW + w] = o;
        }
  return 0;
}

/*
 * Lookup-table sum (Section 7, production model; appendix listing 2LUT, one
 * of its two statements):
 *     O(i,j) +=! LUT(Idx(i,k), j)
 * LUT is [E,D] fp32, Idx is [B,L] int32, O is [B,D].  i and j range over the
 * rows of Idx and the columns of LUT, k over the columns of Idx; an index
 * that occurs several times in a row counts as often.  The comprehension
 * gives no meaning to an index outside [0,E): the evaluator checks all of
 * them first and returns 3 without writing anything.
 */
int tc_oracle_lut(const float *LUT, const int32_t *Idx, double *O, int64_t E,
                  int64_t D, int64_t B, int64_t L) {
  if (!LUT || !Idx || !O) return 1;
  if (E <= 0 || D <= 0 || B < 0 || L <= 0) return 2;
  for (int64_t t = 0; t < B * L; t++)
    if (Idx[t] < 0 || (int64_t)Idx[t] >= E) return 3;
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int64_t i = 0; i < B; i++)
    for (int64_t j = 0; j < D; j++) {
      double o = 0.0; /* "+=!" */
      for (int64_t k = 0; k < L; k++)
        o += (double)LUT[(int64_t)Idx[i * L + k] * D + j];
      O[i * D + j] = o;
    }
  return 0;
}
