/*
 * CPU oracle for the block-sparse MLP path of BLaST (arxiv 2507.03117).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, written to be checked against the
 * paper by eye.  It shares no code with the HIP library, is never called by the
 * product path, and exists so that GPU results can be compared with something
 * independent.  Callers: the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg.
 *
 * What it computes (all pointers are HOST pointers):
 *   - block scores  = squared Frobenius norm of each b x b block  (Sec. 3.2)
 *   - block mask    = keep the highest-scoring blocks until the requested
 *                     sparsity is reached                           (Sec. 3.2)
 *   - packing       = row-pointer / column-index / block-value arrays of the
 *                     masked weight (BSR of the out x in weight, which is the
 *                     paper's BCSC of its transposed weight)  (Sec. 3.2, 3.4.1)
 *   - SpMM          = Y = W~ X with W~ the dense masked weight; the kernel of
 *                     Sec. 3.4 only skips blocks that are absent, i.e. it reaches
 *                     exactly this dense result, so the oracle is the definition:
 *                     expand to dense, naive triple loop, fp64.
 *   - MLP           = Eq. (1): Y = W~down ( act(W~gate X) (.) (W~up X) ), with the
 *                     intermediate H rounded once to bf16 (the precision in which
 *                     it enters the second contraction on the device); the two-matrix
 *                     form Y = W~2 act(W~1 X) of Sec. 2.1 with the same rounding.
 *   - backward      = dX = W~^T dY and the gradient of the stored blocks, the entries
 *                     of dY X^T on kept blocks (Sec. 3.2: one pruned matrix for
 *                     forward and backward).
 *   - mask update   = one generate_masks() round of blocked prune-and-grow and the
 *                     cubic sparsity schedule, Eq. (2) (Sec. 3.2); block scores by
 *                     2D average pooling of a sensitivity matrix (Sec. 3.3).
 *   - E5M2          = the 8-bit floating-point type of Sec. 5.2: exact decode,
 *                     round-to-nearest-even encode, the product on E5M2 operands.
 * Every function is pinned by tests that do not go through the HIP library
 * (closed forms, library routines, exact rational brute force, invariants); none
 * is "parity unpinned".
 *
 * Readings of points the paper leaves open (kept identical in the HIP library
 * by specification, not by shared code):
 *   - number of dropped blocks for sparsity s over N blocks: ceil(s*N), computed
 *     in integers on basis points: s_bp = round(s*1e4), n_zero = ceil(s_bp*N/1e4).
 *   - ranking by the squared norm in fp64; ties broken by the lower linear block
 *     index (block_row * NBc + block_col) being kept first.
 *   - a kept block is stored even if all its values are zero.
 *
 * OpenMP is used only to run independent output rows on several cores; every
 * individual sum is a sequential fp64 loop in index order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_f64(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* fp32 -> bf16, round to nearest even (no NaN handling needed for finite data). */
static inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Sec. 3.2: the lowest-scoring blocks go until the zero fraction reaches s. */
int64_t oracle_n_keep(int64_t n_blocks, double sparsity) {
  int64_t s_bp = (int64_t)llround(sparsity * 10000.0);
  int64_t n_zero = (s_bp * n_blocks + 9999) / 10000;
  if (n_zero > n_blocks) n_zero = n_blocks;
  if (n_zero < 0) n_zero = 0;
  return n_blocks - n_zero;
}

/* Sec. 3.2: each b x b block is scored by its Frobenius norm; we rank by the
 * square (same order, no sqrt).  Sum in row-major order inside the block. */
void oracle_block_scores(const uint16_t* W, int64_t ldw, int64_t rows, int64_t cols, int32_t b,
                         double* score /* [rows/b][cols/b] */) {
  int64_t nbr = rows / b, nbc = cols / b;
  for (int64_t br = 0; br < nbr; ++br)
    for (int64_t bc = 0; bc < nbc; ++bc) {
      double s = 0.0;
      for (int32_t i = 0; i < b; ++i)
        for (int32_t j = 0; j < b; ++j) {
          double w = bf16_to_f64(W[(br * b + i) * ldw + bc * b + j]);
          s += w * w;
        }
      score[br * nbc + bc] = s;
    }
}

typedef struct {
  double score;
  int64_t idx;
} scored_t;

static int cmp_scored(const void* pa, const void* pb) {
  const scored_t* a = (const scored_t*)pa;
  const scored_t* b = (const scored_t*)pb;
  if (a->score > b->score) return -1; /* higher score first */
  if (a->score < b->score) return 1;
  if (a->idx < b->idx) return -1; /* then lower index first */
  if (a->idx > b->idx) return 1;
  return 0;
}

/* Full sort of (score desc, index asc); keep the first n_keep.  Returns n_keep.
 * gap_out (may be NULL) receives the relative gap between the last kept and the
 * first dropped score, so a test can reject inputs whose selection hangs on
 * rounding. */
int64_t oracle_topk_mask(const double* score, int64_t n_blocks, double sparsity, uint8_t* mask, double* gap_out) {
  int64_t n_keep = oracle_n_keep(n_blocks, sparsity);
  scored_t* a = (scored_t*)malloc(sizeof(scored_t) * (size_t)(n_blocks > 0 ? n_blocks : 1));
  for (int64_t i = 0; i < n_blocks; ++i) {
    a[i].score = score[i];
    a[i].idx = i;
  }
  qsort(a, (size_t)n_blocks, sizeof(scored_t), cmp_scored);
  memset(mask, 0, (size_t)n_blocks);
  for (int64_t i = 0; i < n_keep; ++i) mask[a[i].idx] = 1;
  if (gap_out) {
    /* relative to the larger magnitude of the two, so that it also means something for negative scores
     * (pooled sensitivities may have any sign); identical for the non-negative Frobenius scores */
    double den = 0.0;
    if (n_keep > 0 && n_keep < n_blocks) den = fmax(fabs(a[n_keep - 1].score), fabs(a[n_keep].score));
    if (den > 0.0)
      *gap_out = (a[n_keep - 1].score - a[n_keep].score) / den;
    else
      *gap_out = 1.0;
  }
  free(a);
  return n_keep;
}

/* Sec. 3.2 / 3.4.1: compressed block format of W (.) mask.  For each block row in
 * order, the kept block columns in ascending order; block values row-major, raw
 * bf16 bit patterns.  row_order = block rows by stored-block count, descending,
 * stable (the load-balance schedule).  Returns nnz. */
int64_t oracle_pack(const uint16_t* W, int64_t ldw, int64_t rows, int64_t cols, int32_t b, const uint8_t* mask,
                    int32_t* row_ptr, int32_t* col_idx, uint16_t* vals, int32_t* row_order) {
  int64_t nbr = rows / b, nbc = cols / b, nnz = 0;
  row_ptr[0] = 0;
  for (int64_t br = 0; br < nbr; ++br) {
    for (int64_t bc = 0; bc < nbc; ++bc) {
      if (!mask[br * nbc + bc]) continue;
      if (col_idx) col_idx[nnz] = (int32_t)bc;
      if (vals)
        for (int32_t i = 0; i < b; ++i)
          for (int32_t j = 0; j < b; ++j) /* mask code 2: a regrown block, stored with zero values (Sec. 3.2) */
            vals[(nnz * b + i) * b + j] = mask[br * nbc + bc] == 2 ? 0 : W[(br * b + i) * ldw + bc * b + j];
      ++nnz;
    }
    row_ptr[br + 1] = (int32_t)nnz;
  }
  if (row_order) {
    /* stable insertion sort by count descending */
    for (int64_t r = 0; r < nbr; ++r) {
      int32_t cnt = row_ptr[r + 1] - row_ptr[r];
      int64_t p = r;
      while (p > 0) {
        int32_t q = row_order[p - 1];
        if (row_ptr[q + 1] - row_ptr[q] >= cnt) break;
        row_order[p] = q;
        --p;
      }
      row_order[p] = (int32_t)r;
    }
  }
  return nnz;
}

/* Inverse of oracle_pack: dense rows x cols matrix of bf16 bit patterns, zero
 * (bit pattern 0) outside stored blocks. */
void oracle_unpack(int64_t rows, int64_t cols, int32_t b, const int32_t* row_ptr, const int32_t* col_idx,
                   const uint16_t* vals, uint16_t* Wd /* [rows][cols] */) {
  int64_t nbr = rows / b;
  memset(Wd, 0, sizeof(uint16_t) * (size_t)rows * (size_t)cols);
  for (int64_t br = 0; br < nbr; ++br)
    for (int64_t k = row_ptr[br]; k < row_ptr[br + 1]; ++k) {
      int64_t bc = col_idx[k];
      for (int32_t i = 0; i < b; ++i)
        for (int32_t j = 0; j < b; ++j) Wd[(br * b + i) * cols + bc * b + j] = vals[(k * b + i) * b + j];
    }
}

/* Y[i][t] = sum_k Wd[i][k] * X(k,t), fp64, k ascending.  X element (k,t) lives at
 * X[k*sxk + t*sxt].  Y is [rows][T] row-major fp64. */
static void dense_matmul_bf16(const uint16_t* Wd, int64_t rows, int64_t cols, const uint16_t* X, int64_t sxk,
                              int64_t sxt, int64_t T, double* Y) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t t = 0; t < T; ++t) {
      double s = 0.0;
      for (int64_t k = 0; k < cols; ++k) s += bf16_to_f64(Wd[i * cols + k]) * bf16_to_f64(X[k * sxk + t * sxt]);
      Y[i * T + t] = s;
    }
}

/* Sec. 3.4: block-sparse Y = W X, as the dense masked product. */
void oracle_spmm(int64_t rows, int64_t cols, int32_t b, const int32_t* row_ptr, const int32_t* col_idx,
                 const uint16_t* vals, const uint16_t* X, int64_t sxk, int64_t sxt, int64_t T,
                 double* Y /* [rows][T] */) {
  uint16_t* Wd = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)rows * (size_t)cols);
  oracle_unpack(rows, cols, b, row_ptr, col_idx, vals, Wd);
  dense_matmul_bf16(Wd, rows, cols, X, sxk, sxt, T, Y);
  free(Wd);
}

/* The same contraction with fp32 accumulators: bounds what fp32 accumulation
 * (the device's precision) can cost relative to the fp64 result. */
void oracle_spmm_f32acc(int64_t rows, int64_t cols, int32_t b, const int32_t* row_ptr, const int32_t* col_idx,
                        const uint16_t* vals, const uint16_t* X, int64_t sxk, int64_t sxt, int64_t T,
                        double* Y /* [rows][T] */) {
  uint16_t* Wd = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)rows * (size_t)cols);
  oracle_unpack(rows, cols, b, row_ptr, col_idx, vals, Wd);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t t = 0; t < T; ++t) {
      float s = 0.0f;
      for (int64_t k = 0; k < cols; ++k)
        s += (float)bf16_to_f64(Wd[i * cols + k]) * (float)bf16_to_f64(X[k * sxk + t * sxt]);
      Y[i * T + t] = (double)s;
    }
  free(Wd);
}

/* activation codes: 0 = SiLU (x * sigmoid(x)), 1 = GELU (erf form), 2 = ReLU */
double oracle_act(int32_t act, double g) {
  switch (act) {
    case 0: return g / (1.0 + exp(-g));
    case 1: return 0.5 * g * (1.0 + erf(g / sqrt(2.0)));
    case 2: return g > 0.0 ? g : 0.0;
    default: return NAN;
  }
}

/* Eq. (1) with weights stored out x in:  G = W~g X, U = W~u X, H = bf16(act(G) * U),
 * Y = W~d H.  E = hidden, I = intermediate.  gate/up are I x E, down is E x I.
 * H_bits (may be NULL) receives the rounded intermediate, [I][T]. */
void oracle_mlp(int64_t E, int64_t I, int32_t b,
                const int32_t* g_row_ptr, const int32_t* g_col_idx, const uint16_t* g_vals,
                const int32_t* u_row_ptr, const int32_t* u_col_idx, const uint16_t* u_vals,
                const int32_t* d_row_ptr, const int32_t* d_col_idx, const uint16_t* d_vals,
                const uint16_t* X, int64_t sxk, int64_t sxt, int64_t T, int32_t act,
                double* Y /* [E][T] */, uint16_t* H_bits /* [I][T] or NULL */) {
  size_t it = (size_t)I * (size_t)T;
  double* G = (double*)malloc(sizeof(double) * (it ? it : 1));
  double* U = (double*)malloc(sizeof(double) * (it ? it : 1));
  uint16_t* H = (uint16_t*)malloc(sizeof(uint16_t) * (it ? it : 1));
  oracle_spmm(I, E, b, g_row_ptr, g_col_idx, g_vals, X, sxk, sxt, T, G);
  oracle_spmm(I, E, b, u_row_ptr, u_col_idx, u_vals, X, sxk, sxt, T, U);
  for (size_t p = 0; p < it; ++p) {
    double h = oracle_act(act, G[p]) * U[p];
    H[p] = f32_to_bf16_rne((float)h); /* fp64 -> fp32 (RNE) -> bf16 (RNE) */
  }
  /* H is [I][T] row-major: element (k = i, t) at H[i*T + t] */
  oracle_spmm(E, I, b, d_row_ptr, d_col_idx, d_vals, H, T, 1, T, Y);
  if (H_bits) memcpy(H_bits, H, sizeof(uint16_t) * it);
  free(G);
  free(U);
  free(H);
}

/* Two-matrix MLP (Sec. 2.1: two or three weight matrices; Sec. 3.4.3: two projections with an element-wise
 * nonlinearity in between), weights stored out x in:  G = W~1 X, H = bf16(act(G)), Y = W~2 H.
 * W1 is I x E, W2 is E x I.  H_bits (may be NULL) receives the rounded intermediate, [I][T]. */
void oracle_mlp2(int64_t E, int64_t I, int32_t b,
                 const int32_t* w1_row_ptr, const int32_t* w1_col_idx, const uint16_t* w1_vals,
                 const int32_t* w2_row_ptr, const int32_t* w2_col_idx, const uint16_t* w2_vals,
                 const uint16_t* X, int64_t sxk, int64_t sxt, int64_t T, int32_t act,
                 double* Y /* [E][T] */, uint16_t* H_bits /* [I][T] or NULL */) {
  size_t it = (size_t)I * (size_t)T;
  double* G = (double*)malloc(sizeof(double) * (it ? it : 1));
  uint16_t* H = (uint16_t*)malloc(sizeof(uint16_t) * (it ? it : 1));
  oracle_spmm(I, E, b, w1_row_ptr, w1_col_idx, w1_vals, X, sxk, sxt, T, G);
  for (size_t p = 0; p < it; ++p) H[p] = f32_to_bf16_rne((float)oracle_act(act, G[p]));
  oracle_spmm(E, I, b, w2_row_ptr, w2_col_idx, w2_vals, H, T, 1, T, Y);
  if (H_bits) memcpy(H_bits, H, sizeof(uint16_t) * it);
  free(G);
  free(H);
}

/* ---- backward pass on the same pruned weight (Sec. 3.2: the pruned matrix is the one used in forward and
 * backward propagation; Sec. 3.4: the product with the sparse matrix on the other side is the symmetric
 * kernel).  With Y = W~ X:  dX = W~^T dY  and  dW~ = dY X^T on the kept blocks (a dropped block holds no
 * weight, so it receives no gradient). ---- */

/* dX[k][t] = sum_i Wd[i][k] * dY(i,t), fp64, i ascending: the dense masked definition.  dY element (i,t)
 * lives at dY[i*syi + t*syt].  dX is [cols][T] row-major fp64. */
void oracle_spmm_t(int64_t rows, int64_t cols, int32_t b, const int32_t* row_ptr, const int32_t* col_idx,
                   const uint16_t* vals, const uint16_t* dY, int64_t syi, int64_t syt, int64_t T,
                   double* dX /* [cols][T] */) {
  uint16_t* Wd = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)(rows * cols > 0 ? rows * cols : 1));
  oracle_unpack(rows, cols, b, row_ptr, col_idx, vals, Wd);
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < cols; ++k)
    for (int64_t t = 0; t < T; ++t) {
      double s = 0.0;
      for (int64_t i = 0; i < rows; ++i) s += bf16_to_f64(Wd[i * cols + k]) * bf16_to_f64(dY[i * syi + t * syt]);
      dX[k * T + t] = s;
    }
  free(Wd);
}

/* Gradient of the stored blocks: for the q-th stored block, at block row r and block column c,
 *   dvals[q][i][j] = sum_t dY(r*b + i, t) * X(c*b + j, t),  fp64, t ascending
 * i.e. the entries of the dense dY X^T that fall on kept blocks, in storage order. */
void oracle_sddmm(int64_t rows, int64_t cols, int32_t b, const int32_t* row_ptr, const int32_t* col_idx,
                  const uint16_t* dY, int64_t syi, int64_t syt, const uint16_t* X, int64_t sxk, int64_t sxt,
                  int64_t T, double* dvals /* [nnz][b][b] */) {
  (void)cols;
  int64_t nbr = rows / b;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t r = 0; r < nbr; ++r)
    for (int64_t q = row_ptr[r]; q < row_ptr[r + 1]; ++q) {
      int64_t c = col_idx[q];
      for (int32_t i = 0; i < b; ++i)
        for (int32_t j = 0; j < b; ++j) {
          double s = 0.0;
          for (int64_t t = 0; t < T; ++t)
            s += bf16_to_f64(dY[(r * b + i) * syi + t * syt]) * bf16_to_f64(X[(c * b + j) * sxk + t * sxt]);
          dvals[(q * b + i) * b + j] = s;
        }
    }
}

/* ---- one round of the blocked prune-and-grow mask update (Sec. 3.2, the generate_masks() step) ----
 * S(W): the blocks of W that survive pruning to sparsity s (top blocks by Frobenius norm);
 * S(G): the same selection applied to the gradient G;
 * D = S(G) \ S(W): blocks the gradient ranks high but the weight does not - they are regrown.
 * mask[blk] = 1 for blocks of S(W), 2 for blocks of D (kept in the structure, values start at zero), 0 else. */
void oracle_generate_masks(const uint16_t* W, int64_t ldw, const uint16_t* G, int64_t ldg, int64_t rows, int64_t cols,
                           int32_t b, double sparsity, uint8_t* mask /* [rows/b][cols/b] */) {
  int64_t n = (rows / b) * (cols / b);
  double* sw = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  double* sg = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  uint8_t* mw = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
  uint8_t* mg = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
  oracle_block_scores(W, ldw, rows, cols, b, sw);
  oracle_block_scores(G, ldg, rows, cols, b, sg);
  oracle_topk_mask(sw, n, sparsity, mw, NULL);
  oracle_topk_mask(sg, n, sparsity, mg, NULL);
  for (int64_t i = 0; i < n; ++i) mask[i] = mw[i] ? 1 : (mg[i] ? 2 : 0);
  free(sw);
  free(sg);
  free(mw);
  free(mg);
}

/* Eq. (2): s(i) = s_max + (s_init - s_max) * (1 - i / (m - d))^3.  The paper gives no value past i = m - d,
 * where the cube would turn negative and push s above s_max: the iteration is held at the ends of [0, m - d]. */
double oracle_sparsity_schedule(int64_t i, int64_t m, int64_t d, double s_init, double s_max) {
  int64_t span = m - d;
  if (span <= 0) return s_max;
  if (i < 0) i = 0;
  if (i > span) i = span;
  double f = 1.0 - (double)i / (double)span;
  return s_max + (s_init - s_max) * f * f * f;
}

/* ---- block scores from a sensitivity matrix (Sec. 3.3: the per-weight sensitivities form a matrix of the
 * weight's shape, which is cut into b x b blocks; a block's score is the 2D average pooling of its entries;
 * the blocks with the least score are pruned). ---- */

/* score[br][bc] = mean of S over the block, fp64, row-major order inside the block.  S is fp32 [rows][lds]. */
void oracle_pooled_scores(const float* S, int64_t lds, int64_t rows, int64_t cols, int32_t b,
                          double* score /* [rows/b][cols/b] */) {
  int64_t nbr = rows / b, nbc = cols / b;
  for (int64_t br = 0; br < nbr; ++br)
    for (int64_t bc = 0; bc < nbc; ++bc) {
      double s = 0.0;
      for (int32_t i = 0; i < b; ++i)
        for (int32_t j = 0; j < b; ++j) s += (double)S[(br * b + i) * lds + bc * b + j];
      score[br * nbc + bc] = s / ((double)b * (double)b);
    }
}

/* ---- 8-bit floating point (the paper runs its kernel in float8_e5m2 as well: Sec. 5.2) ----
 * E5M2: 1 sign bit, 5 exponent bits (bias 15), 2 mantissa bits; subnormals, infinities and NaN as in IEEE
 * half precision, of which it is the upper byte.  Largest finite value 1.75 * 2^15 = 57344, smallest
 * subnormal 2^-16. */

/* Exact value of a code. */
double oracle_e5m2_to_f64(uint8_t c) {
  int sign = c >> 7, e = (c >> 2) & 31, m = c & 3;
  double v;
  if (e == 31) v = m ? NAN : INFINITY;
  else if (e == 0) v = ldexp((double)m, -16);            /* subnormal: m * 2^-14 * 2^-2 */
  else v = ldexp(1.0 + (double)m / 4.0, e - 15);
  return sign ? -v : v;
}

/* Round to nearest, ties to the code with an even mantissa; magnitudes that round past the largest finite
 * value become infinity (IEEE rounding).  Written on the value, not on bit patterns: scale so that the
 * spacing of representable numbers around |x| is 1, round to an integer with ties to even, rebuild. */
uint8_t oracle_f64_to_e5m2(double x) {
  uint8_t sign = (uint8_t)(signbit(x) ? 0x80 : 0);
  if (isnan(x)) return (uint8_t)(sign | 0x7E);
  double a = fabs(x);
  if (isinf(a)) return (uint8_t)(sign | 0x7C);
  if (a == 0.0) return sign;
  int ex;
  frexp(a, &ex);            /* a = f * 2^ex, f in [0.5, 1)  ->  a in [2^(ex-1), 2^ex) */
  int e = ex - 1;           /* unbiased exponent of a */
  if (e < -14) e = -14;     /* subnormal range shares the spacing of the lowest normal binade */
  double q = ldexp(a, 2 - e);                 /* spacing 2^(e-2) -> 1 */
  double r = nearbyint(q);                    /* default rounding mode: to nearest, ties to even */
  /* r in [0, 8]; r = 8 means the value rounded up into the next binade */
  int64_t n = (int64_t)r;
  int biased = e + 15;                        /* >= 1 */
  if (n < 4) {                                /* subnormal (only possible when e == -14) */
    return (uint8_t)(sign | (uint8_t)n);
  }
  if (n == 8) { n = 4; biased += 1; }
  if (biased >= 31) return (uint8_t)(sign | 0x7C);
  return (uint8_t)(sign | (biased << 2) | (n - 4));
}

void oracle_quantize_e5m2(const float* x, int64_t n, uint8_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_f64_to_e5m2((double)x[i]);
}

/* Y = W~ X with both operands in E5M2: the dense masked product of the decoded values, fp64.  vals8 holds the
 * stored blocks like the bf16 format does ([nnz][b][b], row-major), one byte per value; X element (k,t) lives
 * at X8[k*sxk + t*sxt]. */
void oracle_spmm_e5m2(int64_t rows, int64_t cols, int32_t b, const int32_t* row_ptr, const int32_t* col_idx,
                      const uint8_t* vals8, const uint8_t* X8, int64_t sxk, int64_t sxt, int64_t T,
                      double* Y /* [rows][T] */) {
  int64_t nbr = rows / b;
  double* Wd = (double*)calloc((size_t)(rows * cols > 0 ? rows * cols : 1), sizeof(double));
  for (int64_t br = 0; br < nbr; ++br)
    for (int64_t k = row_ptr[br]; k < row_ptr[br + 1]; ++k)
      for (int32_t i = 0; i < b; ++i)
        for (int32_t j = 0; j < b; ++j)
          Wd[(br * b + i) * cols + (int64_t)col_idx[k] * b + j] = oracle_e5m2_to_f64(vals8[(k * b + i) * b + j]);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t t = 0; t < T; ++t) {
      double s = 0.0;
      for (int64_t k = 0; k < cols; ++k) s += Wd[i * cols + k] * oracle_e5m2_to_f64(X8[k * sxk + t * sxt]);
      Y[i * T + t] = s;
    }
  free(Wd);
}

/* Y = W~ X with the stored block values in E5M2 and the activations in bf16 (weights in the 8-bit type of
 * Sec. 5.2, activations in the 16-bit type: every code is decoded exactly, the dense masked product is taken
 * in fp64).  X element (k,t) lives at X[k*sxk + t*sxt]. */
void oracle_spmm_e5m2w(int64_t rows, int64_t cols, int32_t b, const int32_t* row_ptr, const int32_t* col_idx,
                       const uint8_t* vals8, const uint16_t* X, int64_t sxk, int64_t sxt, int64_t T,
                       double* Y /* [rows][T] */) {
  int64_t nbr = rows / b;
  double* Wd = (double*)calloc((size_t)(rows * cols > 0 ? rows * cols : 1), sizeof(double));
  for (int64_t br = 0; br < nbr; ++br)
    for (int64_t k = row_ptr[br]; k < row_ptr[br + 1]; ++k)
      for (int32_t i = 0; i < b; ++i)
        for (int32_t j = 0; j < b; ++j)
          Wd[(br * b + i) * cols + (int64_t)col_idx[k] * b + j] = oracle_e5m2_to_f64(vals8[(k * b + i) * b + j]);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t t = 0; t < T; ++t) {
      double s = 0.0;
      for (int64_t k = 0; k < cols; ++k) s += Wd[i * cols + k] * bf16_to_f64(X[k * sxk + t * sxt]);
      Y[i * T + t] = s;
    }
  free(Wd);
}

/* Eq. (1) with the three weights stored in E5M2 (Sec. 5.2) and everything else as in oracle_mlp:
 * G = W~g X, U = W~u X from the decoded codes and the bf16 activations, H = bf16(act(G) * U), Y = W~d H.
 * H_bits (may be NULL) receives the rounded intermediate, [I][T]. */
void oracle_mlp_e5m2w(int64_t E, int64_t I, int32_t b,
                      const int32_t* g_row_ptr, const int32_t* g_col_idx, const uint8_t* g_vals8,
                      const int32_t* u_row_ptr, const int32_t* u_col_idx, const uint8_t* u_vals8,
                      const int32_t* d_row_ptr, const int32_t* d_col_idx, const uint8_t* d_vals8,
                      const uint16_t* X, int64_t sxk, int64_t sxt, int64_t T, int32_t act,
                      double* Y /* [E][T] */, uint16_t* H_bits /* [I][T] or NULL */) {
  size_t it = (size_t)I * (size_t)T;
  double* G = (double*)malloc(sizeof(double) * (it ? it : 1));
  double* U = (double*)malloc(sizeof(double) * (it ? it : 1));
  uint16_t* H = (uint16_t*)malloc(sizeof(uint16_t) * (it ? it : 1));
  oracle_spmm_e5m2w(I, E, b, g_row_ptr, g_col_idx, g_vals8, X, sxk, sxt, T, G);
  oracle_spmm_e5m2w(I, E, b, u_row_ptr, u_col_idx, u_vals8, X, sxk, sxt, T, U);
  for (size_t p = 0; p < it; ++p) H[p] = f32_to_bf16_rne((float)(oracle_act(act, G[p]) * U[p]));
  oracle_spmm_e5m2w(E, I, b, d_row_ptr, d_col_idx, d_vals8, H, T, 1, T, Y);
  if (H_bits) memcpy(H_bits, H, sizeof(uint16_t) * it);
  free(G);
  free(U);
  free(H);
}
