/*
 * CPU oracle for the full-batch GCN hot path (MG-GCN, arXiv 2110.08688).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64, written from the paper's
 * equations; it shares no code, header, table or helper with the HIP library
 * and must never be called from the product path.  Only tests, the smoke
 * check and the bench's cpu_baseline leg may load it.
 *
 * What is the plain definition and what is a reading of the paper:
 *   - Every function below is the textbook definition of the operation it
 *     names (CSR product, dense product, ReLU, softmax cross-entropy, chain
 *     rule), evaluated in double precision in index order.  Nothing here is
 *     an approximation, so "parity unpinned" applies to none of them; the
 *     pins are in tests/test_oracle_*.py (dense brute force, closed forms,
 *     scipy / numpy / torch-autograd third opinions, finite differences).
 *   - Readings of points the paper leaves open are marked "Reading:".
 *   - One extension beyond the paper: an epoch whose SpMMs gather a bfloat16 copy of their
 *     dense operand (mggcn_ref_bf16_*, mggcn_ref_epoch_bf16).  The rounding is the IEEE
 *     definition written out and is pinned by hand-worked values, by an exhaustive check
 *     against the neighbour definition and by torch's conversion; the epoch is pinned by a
 *     numpy / scipy re-composition of the same chain.
 *
 * Parallelism: OpenMP over independent output rows (or output columns for the
 * scatter form) only, so every output element is summed in the same order as
 * the serial loop would sum it.
 *
 * Conventions: dense matrices are row-major with a leading dimension (ld),
 * indices are int32, all pointers are host pointers.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_OK 0
#define REF_E_ARG (-1)
#define REF_E_CSR (-2)
#define REF_E_MEM (-3)

enum { REF_NORM_SYM = 0, REF_NORM_MEAN_IN = 1 };
enum { REF_OP_N = 0, REF_OP_T = 1 };
enum { REF_GEMM_FIRST = 0, REF_SPMM_FIRST = 1 };

/* ------------------------------------------------------------------------
 * Pattern checks
 * --------------------------------------------------------------------- */

/* rows sorted strictly ascending, indices in range */
int mggcn_ref_csr_validate(int n_rows, int n_cols, const int32_t* rowptr, const int32_t* colidx) {
  if (n_rows < 0 || n_cols < 0 || !rowptr) return REF_E_ARG;
  if (rowptr[0] != 0) return REF_E_CSR;
  for (int i = 0; i < n_rows; ++i) {
    if (rowptr[i + 1] < rowptr[i]) return REF_E_CSR;
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
      if (colidx[k] < 0 || colidx[k] >= n_cols) return REF_E_CSR;
      if (k > rowptr[i] && colidx[k] <= colidx[k - 1]) return REF_E_CSR;
    }
  }
  return REF_OK;
}

/* ------------------------------------------------------------------------
 * Normalised adjacency (Eq. 1-2 of the paper; Kipf-style self-loops)
 *
 *   A~  = pattern(A) united with the diagonal          (Reading: an existing
 *         (i,i) stays a single entry of weight 1; rows i >= n_cols of a
 *         rectangular block get no diagonal)
 *   SYM : A^_ij = 1 / sqrt(d_i * d_j), d = number of entries in row i of A~
 *         (Reading: for a non-symmetric pattern both factors are row counts;
 *          a rectangular block passes deg_row / deg_col explicitly)
 *   MEAN_IN (Eq. 2): A^_uv = A~_uv / sum_w A~_wv = 1 / (entries in column v)
 *
 * rowptr_out has n_rows+1 entries; colidx_out / val_out need room for
 * nnz_in + min(n_rows, n_cols) entries.  Returns nnz of A~ (>= 0) or an error.
 * --------------------------------------------------------------------- */
int64_t mggcn_ref_csr_normalize(int n_rows, int n_cols, const int32_t* rowptr_in,
                                const int32_t* colidx_in, int mode, const double* deg_row,
                                const double* deg_col, int32_t* rowptr_out, int32_t* colidx_out,
                                double* val_out) {
  if (mggcn_ref_csr_validate(n_rows, n_cols, rowptr_in, colidx_in) != REF_OK) return REF_E_CSR;
  if (mode != REF_NORM_SYM && mode != REF_NORM_MEAN_IN) return REF_E_ARG;
  if (n_rows != n_cols && mode == REF_NORM_SYM && (!deg_row || !deg_col)) return REF_E_ARG;

  /* 1. pattern with diagonal, columns kept ascending */
  int64_t nnz = 0;
  rowptr_out[0] = 0;
  for (int i = 0; i < n_rows; ++i) {
    int placed = (i >= n_cols); /* nothing to place outside the column range */
    for (int32_t k = rowptr_in[i]; k < rowptr_in[i + 1]; ++k) {
      const int32_t j = colidx_in[k];
      if (!placed && j >= i) {
        if (j != i) colidx_out[nnz++] = i;
        placed = 1;
      }
      colidx_out[nnz++] = j;
    }
    if (!placed) colidx_out[nnz++] = i;
    if (nnz > INT32_MAX) return REF_E_ARG;
    rowptr_out[i + 1] = (int32_t)nnz;
  }

  /* 2. degrees as exact integers */
  double* drow = (double*)malloc(sizeof(double) * (size_t)(n_rows > 0 ? n_rows : 1));
  double* dcol = (double*)calloc((size_t)(n_cols > 0 ? n_cols : 1), sizeof(double));
  if (!drow || !dcol) { free(drow); free(dcol); return REF_E_MEM; }
  for (int i = 0; i < n_rows; ++i) drow[i] = (double)(rowptr_out[i + 1] - rowptr_out[i]);
  for (int64_t k = 0; k < nnz; ++k) dcol[colidx_out[k]] += 1.0;

  /* 3. values */
  for (int i = 0; i < n_rows; ++i) {
    for (int32_t k = rowptr_out[i]; k < rowptr_out[i + 1]; ++k) {
      const int32_t j = colidx_out[k];
      if (mode == REF_NORM_SYM) {
        const double di = deg_row ? deg_row[i] : drow[i];
        const double dj = deg_col ? deg_col[j] : drow[j]; /* square: row count of vertex j */
        val_out[k] = 1.0 / sqrt(di * dj);
      } else {
        const double dj = deg_col ? deg_col[j] : dcol[j];
        val_out[k] = 1.0 / dj;
      }
    }
  }
  free(drow);
  free(dcol);
  return nnz;
}

/* Explicit transpose of a CSR matrix; rows of the result have ascending columns. */
int mggcn_ref_csr_transpose(int n_rows, int n_cols, const int32_t* rowptr, const int32_t* colidx,
                            const double* val, int32_t* rowptr_t, int32_t* colidx_t,
                            double* val_t) {
  const int64_t nnz = rowptr[n_rows];
  int32_t* cur = (int32_t*)calloc((size_t)n_cols + 1, sizeof(int32_t));
  if (!cur) return REF_E_MEM;
  for (int64_t k = 0; k < nnz; ++k) cur[colidx[k] + 1]++;
  rowptr_t[0] = 0;
  for (int j = 0; j < n_cols; ++j) rowptr_t[j + 1] = rowptr_t[j] + cur[j + 1];
  for (int j = 0; j < n_cols; ++j) cur[j] = rowptr_t[j];
  for (int i = 0; i < n_rows; ++i) /* ascending i => ascending columns in each result row */
    for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
      const int32_t p = cur[colidx[k]]++;
      colidx_t[p] = i;
      val_t[p] = val[k];
    }
  free(cur);
  return REF_OK;
}

/* ------------------------------------------------------------------------
 * SpMM (Eq. 6 forward, Eq. 9 backward):  Y = op(A^) * X + beta * Y
 *   op = N :  Y[i,f] = sum_k val[k] * X[colidx[k], f]   over row i, CSR order
 *   op = T :  Y[j,f] = sum_{(i,j)} val_ij * X[i, f]      scatter, ascending i
 * A^ is n_rows x n_cols.  For op N, X has n_cols rows and Y n_rows rows; for
 * op T the other way round.
 * --------------------------------------------------------------------- */
int mggcn_ref_spmm(int op, int n_rows, int n_cols, const int32_t* rowptr, const int32_t* colidx,
                   const double* val, const double* X, int64_t ldx, int F, double beta, double* Y,
                   int64_t ldy) {
  if (F < 0 || ldx < F || ldy < F) return REF_E_ARG;
  const int out_rows = (op == REF_OP_N) ? n_rows : n_cols;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < out_rows; ++i)
    for (int f = 0; f < F; ++f) Y[i * ldy + f] = (beta == 0.0) ? 0.0 : beta * Y[i * ldy + f];

  if (op == REF_OP_N) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int i = 0; i < n_rows; ++i)
      for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
        const double a = val[k];
        const double* x = X + (int64_t)colidx[k] * ldx;
        for (int f = 0; f < F; ++f) Y[i * ldy + f] += a * x[f];
      }
  } else {
    /* each thread owns a band of feature columns, so the scatter is race-free
       and every Y[j,f] is accumulated in ascending i exactly as written above */
#pragma omp parallel
    {
      int nt = 1, t = 0;
#ifdef _OPENMP
      nt = omp_get_num_threads();
      t = omp_get_thread_num();
#endif
      const int f0 = (int)((int64_t)F * t / nt), f1 = (int)((int64_t)F * (t + 1) / nt);
      if (f1 > f0)
        for (int i = 0; i < n_rows; ++i)
          for (int32_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
            const double a = val[k];
            double* y = Y + (int64_t)colidx[k] * ldy;
            const double* x = X + (int64_t)i * ldx;
            for (int f = f0; f < f1; ++f) y[f] += a * x[f];
          }
    }
  }
  return REF_OK;
}

/* ------------------------------------------------------------------------
 * Lower-precision gathered operand: the dense operand of an SpMM held as bfloat16 (sign, 8
 * exponent bits, 7 fraction bits: a float32 whose low 16 bits are zero), products and sums
 * still exact here.  This is an extension beyond the paper, which keeps everything in fp32.
 *
 * Rounding float32 -> bfloat16 is IEEE round-to-nearest, ties to even, written out as its
 * definition: take the two bfloat16 neighbours of x (toward zero and away from zero), return
 * the nearer one, and on a tie the one whose last fraction bit is 0.  A value at least half a
 * step above the largest finite bfloat16 goes to infinity; a NaN stays a NaN.
 * --------------------------------------------------------------------- */
static float f32_from_bits(uint32_t u) { float f; memcpy(&f, &u, sizeof f); return f; }

uint16_t mggcn_ref_bf16_code(float x) {
  uint32_t u;
  memcpy(&u, &x, sizeof u);
  if ((u & 0x7F800000u) == 0x7F800000u) {            /* infinity or NaN */
    if (u & 0x007FFFFFu) return (uint16_t)((u >> 16) | 0x0040u); /* keep a NaN a (quiet) NaN */
    return (uint16_t)(u >> 16);
  }
  const uint32_t lo = u & 0xFFFF0000u;                /* neighbour toward zero */
  if (lo == u) return (uint16_t)(u >> 16);            /* already representable */
  const uint32_t hi = lo + 0x00010000u;               /* neighbour away from zero */
  const double ax = fabs((double)x);
  const double alo = fabs((double)f32_from_bits(lo));
  /* beyond the largest finite value the next step of the same size is 2^128 */
  const double ahi = ((hi & 0x7FFFFFFFu) == 0x7F800000u) ? ldexp(1.0, 128) : fabs((double)f32_from_bits(hi));
  const double below = ax - alo, above = ahi - ax;    /* both exact in double */
  if (below < above) return (uint16_t)(lo >> 16);
  if (above < below) return (uint16_t)(hi >> 16);
  return (uint16_t)((((lo >> 16) & 1u) == 0u ? lo : hi) >> 16);
}

float mggcn_ref_bf16_value(uint16_t code) { return f32_from_bits((uint32_t)code << 16); }

/* codes_out / values_out may each be NULL */
void mggcn_ref_bf16_round(int64_t count, const float* in, uint16_t* codes_out, float* values_out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    const uint16_t c = mggcn_ref_bf16_code(in[i]);
    if (codes_out) codes_out[i] = c;
    if (values_out) values_out[i] = mggcn_ref_bf16_value(c);
  }
}

/* What one SpMM of a chain does about its operand.  bf16 == 0: nothing (the fp32 path).
   Otherwise the rows x F operand is replaced, before the product, by
     inject != NULL : the bfloat16 codes handed in (dense, ld = F).  Used for chain-level parity:
                      which neighbour a value within rounding of a tie goes to is a discrete
                      decision, comparable only when both sides take it from the same numbers
                      (the device's fp32 values);
     inject == NULL : the oracle's own value, rounded to float32 and then to bfloat16.
   record != NULL receives the oracle's own codes either way, so that a test can see how far
   the injected ones are from them. */
typedef struct {
  int bf16;
  const uint16_t* inject;
  uint16_t* record;
} RefGather;

static int spmm_gathered(const RefGather* q, int op, int n_rows, int n_cols, const int32_t* rowptr,
                         const int32_t* colidx, const double* val, const double* X, int64_t ldx, int F,
                         double* Y, int64_t ldy) {
  if (!q || !q->bf16) return mggcn_ref_spmm(op, n_rows, n_cols, rowptr, colidx, val, X, ldx, F, 0.0, Y, ldy);
  const int64_t rows = (op == REF_OP_N) ? n_cols : n_rows;
  double* Xq = (double*)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * (size_t)(F > 0 ? F : 1));
  if (!Xq) return REF_E_MEM;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int f = 0; f < F; ++f) {
      const uint16_t own = mggcn_ref_bf16_code((float)X[i * ldx + f]);
      if (q->record) q->record[i * F + f] = own;
      Xq[i * F + f] = (double)mggcn_ref_bf16_value(q->inject ? q->inject[i * F + f] : own);
    }
  const int rc = mggcn_ref_spmm(op, n_rows, n_cols, rowptr, colidx, val, Xq, F, F, 0.0, Y, ldy);
  free(Xq);
  return rc;
}

/* ------------------------------------------------------------------------
 * GeMM (Eq. 5, 10, 11):  C = op(A) * op(B) + beta * C,  C is M x N, inner K.
 *   opA = N: A is M x K;  opA = T: A is K x M (used as its transpose)
 *   opB = N: B is K x N;  opB = T: B is N x K
 * --------------------------------------------------------------------- */
int mggcn_ref_gemm(int opA, int opB, int M, int N, int K, const double* A, int64_t lda,
                   const double* B, int64_t ldb, double beta, double* C, int64_t ldc) {
  if (M < 0 || N < 0 || K < 0 || ldc < N) return REF_E_ARG;
#pragma omp parallel for schedule(static)
  for (int m = 0; m < M; ++m) {
    double* c = C + (int64_t)m * ldc;
    for (int n = 0; n < N; ++n) c[n] = (beta == 0.0) ? 0.0 : beta * c[n];
    for (int k = 0; k < K; ++k) {
      const double a = (opA == REF_OP_N) ? A[(int64_t)m * lda + k] : A[(int64_t)k * lda + m];
      if (opB == REF_OP_N) {
        const double* b = B + (int64_t)k * ldb;
        for (int n = 0; n < N; ++n) c[n] += a * b[n];
      } else {
        for (int n = 0; n < N; ++n) c[n] += a * B[(int64_t)n * ldb + k];
      }
    }
  }
  return REF_OK;
}

/* ReLU (Eq. 7) in place */
void mggcn_ref_relu(int64_t rows, int cols, double* Z, int64_t ld) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int f = 0; f < cols; ++f)
      if (!(Z[i * ld + f] > 0.0)) Z[i * ld + f] = 0.0;
}

/* ReLU' (Eq. 8): G <- G where act > 0, else 0.  Reading: derivative 0 at act <= 0;
   act may be the pre- or the post-activation value (same mask). */
void mggcn_ref_relu_bwd(int64_t rows, int cols, const double* act, int64_t lda, double* G,
                        int64_t ldg) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int f = 0; f < cols; ++f)
      if (!(act[i * lda + f] > 0.0)) G[i * ldg + f] = 0.0;
}

/* ReLU' with the 0/1 decisions handed in (dense rows x cols bytes) instead of being taken
   from fp64 activations.  Used for epoch-level parity: whether an activation that is zero to
   within rounding counts as "on" is a discrete decision, and a comparison is only meaningful
   when both sides take it from the same numbers (here: the fp32 activations of the device). */
void mggcn_ref_apply_mask(int64_t rows, int cols, const uint8_t* mask, double* G, int64_t ldg) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int f = 0; f < cols; ++f)
      if (!mask[i * cols + f]) G[i * ldg + f] = 0.0;
}

/* Softmax cross-entropy, mean over all n rows (Reading: every vertex is labelled,
   no mask), and its gradient dZ = (softmax(Z) - onehot) / n.  dZ may alias Z. */
int mggcn_ref_softmax_ce(int64_t n, int C, const double* Z, int64_t ldz, const int32_t* labels,
                         double* loss_out, double* dZ, int64_t ldd) {
  if (n <= 0 || C <= 0) return REF_E_ARG;
  double total = 0.0;
  for (int64_t i = 0; i < n; ++i) { /* serial: one fixed summation order for the mean */
    const double* z = Z + i * ldz;
    if (labels[i] < 0 || labels[i] >= C) return REF_E_ARG;
    double mx = z[0];
    for (int c = 1; c < C; ++c) if (z[c] > mx) mx = z[c];
    double s = 0.0;
    for (int c = 0; c < C; ++c) s += exp(z[c] - mx);
    const double lse = mx + log(s);
    total += lse - z[labels[i]];
    if (dZ) {
      for (int c = 0; c < C; ++c) {
        const double p = exp(z[c] - lse);
        dZ[i * ldd + c] = (p - (c == labels[i] ? 1.0 : 0.0)) / (double)n;
      }
    }
  }
  if (loss_out) *loss_out = total / (double)n;
  return REF_OK;
}

/* Order rule ("Order of Computation"): SpMM first iff d_in < d_out; tie -> GeMM first. */
int mggcn_ref_order(int d_in, int d_out) { return d_in < d_out ? REF_SPMM_FIRST : REF_GEMM_FIRST; }

static double* dalloc(int64_t rows, int64_t cols) {
  return (double*)calloc((size_t)(rows > 0 ? rows : 1) * (size_t)(cols > 0 ? cols : 1), sizeof(double));
}

/* ------------------------------------------------------------------------
 * One layer forward (Eq. 5-7):  H_out = act( A^ * H_in * W )
 *   order GEMM_FIRST:  HW = H_in*W ; Z = A^*HW
 *   order SPMM_FIRST:  P  = A^*H_in ; Z = P*W
 * A^ is n x n here (square graph), op N.  relu != 0 applies Eq. 7.
 * --------------------------------------------------------------------- */
static int layer_fwd_impl(int n, const int32_t* rowptr, const int32_t* colidx, const double* val,
                          int d_in, int d_out, int order, int relu, const double* H_in, int64_t ldh,
                          const double* W, int64_t ldw, double* H_out, int64_t ldo, const RefGather* q) {
  int rc;
  if (order == REF_GEMM_FIRST) {
    double* HW = dalloc(n, d_out);
    if (!HW) return REF_E_MEM;
    rc = mggcn_ref_gemm(REF_OP_N, REF_OP_N, n, d_out, d_in, H_in, ldh, W, ldw, 0.0, HW, d_out);
    if (!rc) rc = spmm_gathered(q, REF_OP_N, n, n, rowptr, colidx, val, HW, d_out, d_out, H_out, ldo);
    free(HW);
  } else {
    double* P = dalloc(n, d_in);
    if (!P) return REF_E_MEM;
    rc = spmm_gathered(q, REF_OP_N, n, n, rowptr, colidx, val, H_in, ldh, d_in, P, d_in);
    if (!rc) rc = mggcn_ref_gemm(REF_OP_N, REF_OP_N, n, d_out, d_in, P, d_in, W, ldw, 0.0, H_out, ldo);
    free(P);
  }
  if (!rc && relu) mggcn_ref_relu(n, d_out, H_out, ldo);
  return rc;
}

int mggcn_ref_layer_fwd(int n, const int32_t* rowptr, const int32_t* colidx, const double* val,
                        int d_in, int d_out, int order, int relu, const double* H_in, int64_t ldh,
                        const double* W, int64_t ldw, double* H_out, int64_t ldo) {
  return layer_fwd_impl(n, rowptr, colidx, val, d_in, d_out, order, relu, H_in, ldh, W, ldw, H_out, ldo, NULL);
}

/* ------------------------------------------------------------------------
 * One layer backward (Eq. 8-11), exact chain rule for Z = A^ * H_in * W:
 *   Z_G = G (.) 1[H_out > 0]   if the layer had a ReLU, else Z_G = G
 *   W_G = H_in^T * (A^^T * Z_G)           (Reading of Eq. 10: shaped like W)
 *   H_G = (A^^T * Z_G) * W^T              (Eq. 9, 11)
 * Both operation orders give the same derivative; `order` picks which
 * association is evaluated so that both can be checked against each other:
 *   GEMM_FIRST:  T = A^^T Z_G ; W_G = H_in^T T ; H_G = T W^T
 *   SPMM_FIRST:  P = A^ H_in ; W_G = P^T Z_G ; U = Z_G W^T ; H_G = A^^T U
 * G is overwritten by Z_G.  H_G may be NULL (first layer: no input gradient).
 * --------------------------------------------------------------------- */
static int layer_bwd_impl(int n, const int32_t* rowptr, const int32_t* colidx, const double* val,
                          int d_in, int d_out, int order, int relu, const double* H_in, int64_t ldh,
                          const double* H_out, int64_t ldo, double* G, int64_t ldg, const double* W,
                          int64_t ldw, double* W_G, int64_t ldwg, double* H_G, int64_t ldhg,
                          const RefGather* q_fwd /* the layer's forward SpMM, redone for P */,
                          const RefGather* q_bwd /* its backward SpMM */) {
  int rc = REF_OK;
  if (relu) mggcn_ref_relu_bwd(n, d_out, H_out, ldo, G, ldg);
  if (order == REF_GEMM_FIRST) {
    double* T = dalloc(n, d_out);
    if (!T) return REF_E_MEM;
    rc = spmm_gathered(q_bwd, REF_OP_T, n, n, rowptr, colidx, val, G, ldg, d_out, T, d_out);
    if (!rc) rc = mggcn_ref_gemm(REF_OP_T, REF_OP_N, d_in, d_out, n, H_in, ldh, T, d_out, 0.0, W_G, ldwg);
    if (!rc && H_G) rc = mggcn_ref_gemm(REF_OP_N, REF_OP_T, n, d_in, d_out, T, d_out, W, ldw, 0.0, H_G, ldhg);
    free(T);
  } else {
    double* P = dalloc(n, d_in);
    if (!P) return REF_E_MEM;
    rc = spmm_gathered(q_fwd, REF_OP_N, n, n, rowptr, colidx, val, H_in, ldh, d_in, P, d_in);
    if (!rc) rc = mggcn_ref_gemm(REF_OP_T, REF_OP_N, d_in, d_out, n, P, d_in, G, ldg, 0.0, W_G, ldwg);
    free(P);
    if (!rc && H_G) {
      double* U = dalloc(n, d_in);
      if (!U) return REF_E_MEM;
      rc = mggcn_ref_gemm(REF_OP_N, REF_OP_T, n, d_in, d_out, G, ldg, W, ldw, 0.0, U, d_in);
      if (!rc) rc = spmm_gathered(q_bwd, REF_OP_T, n, n, rowptr, colidx, val, U, d_in, d_in, H_G, ldhg);
      free(U);
    }
  }
  return rc;
}

int mggcn_ref_layer_bwd(int n, const int32_t* rowptr, const int32_t* colidx, const double* val,
                        int d_in, int d_out, int order, int relu, const double* H_in, int64_t ldh,
                        const double* H_out, int64_t ldo, double* G, int64_t ldg, const double* W,
                        int64_t ldw, double* W_G, int64_t ldwg, double* H_G, int64_t ldhg) {
  return layer_bwd_impl(n, rowptr, colidx, val, d_in, d_out, order, relu, H_in, ldh, H_out, ldo, G, ldg, W, ldw,
                        W_G, ldwg, H_G, ldhg, NULL, NULL);
}

/* ------------------------------------------------------------------------
 * One epoch without optimiser: L forward layers, softmax-CE, L backward layers.
 *   dims[0..L]  layer widths;  W[l] is dims[l] x dims[l+1], dense (ld = dims[l+1])
 *   orders[l]   operation order per layer, or NULL for the paper's rule
 *   Reading: no ReLU on the last layer (its output are the logits).
 *   relu_masks  NULL, or L-1 dense byte matrices (n x dims[l+1]) with the ReLU' decisions of
 *               the hidden layers to use in the backward pass instead of the oracle's own
 *               (see mggcn_ref_apply_mask); the forward pass always uses Eq. 7 as is.
 * Outputs: *loss, W_G[l] (same shapes as W[l]); logits_out (n x dims[L]) optional.
 * --------------------------------------------------------------------- */
static int epoch_impl(int n, const int32_t* rowptr, const int32_t* colidx, const double* val, int L,
                      const int32_t* dims, const int32_t* orders, const double* X, int64_t ldx,
                      const int32_t* labels, const double* const* W, double* loss, double* const* W_G,
                      double* logits_out, const uint8_t* const* relu_masks, int bf16,
                      const uint16_t* const* fwd_in, const uint16_t* const* bwd_in,
                      uint16_t* const* fwd_out, uint16_t* const* bwd_out) {
  if (L < 1) return REF_E_ARG;
  int rc = REF_OK;
  double** H = (double**)calloc((size_t)L + 1, sizeof(double*)); /* H[l] = input of layer l */
  if (!H) return REF_E_MEM;
  H[0] = (double*)X;
  for (int l = 0; l < L && !rc; ++l) {
    H[l + 1] = dalloc(n, dims[l + 1]);
    if (!H[l + 1]) { rc = REF_E_MEM; break; }
    const int ord = orders ? orders[l] : mggcn_ref_order(dims[l], dims[l + 1]);
    const RefGather q = {bf16, fwd_in ? fwd_in[l] : NULL, fwd_out ? fwd_out[l] : NULL};
    rc = layer_fwd_impl(n, rowptr, colidx, val, dims[l], dims[l + 1], ord, l + 1 < L,
                        l == 0 ? X : H[l], l == 0 ? ldx : dims[l], W[l], dims[l + 1], H[l + 1],
                        dims[l + 1], &q);
  }
  double* G = NULL;
  if (!rc) {
    if (logits_out) memcpy(logits_out, H[L], sizeof(double) * (size_t)n * (size_t)dims[L]);
    G = dalloc(n, dims[L]);
    if (!G) rc = REF_E_MEM;
  }
  if (!rc) rc = mggcn_ref_softmax_ce(n, dims[L], H[L], dims[L], labels, loss, G, dims[L]);
  for (int l = L - 1; l >= 0 && !rc; --l) {
    const int ord = orders ? orders[l] : mggcn_ref_order(dims[l], dims[l + 1]);
    double* HG = (l > 0) ? dalloc(n, dims[l]) : NULL;
    if (l > 0 && !HG) { rc = REF_E_MEM; break; }
    int own_relu = l + 1 < L;
    if (own_relu && relu_masks) {
      mggcn_ref_apply_mask(n, dims[l + 1], relu_masks[l], G, dims[l + 1]);
      own_relu = 0;
    }
    const RefGather qf = {bf16, fwd_in ? fwd_in[l] : NULL, NULL};
    const RefGather qb = {bf16, bwd_in ? bwd_in[l] : NULL, bwd_out ? bwd_out[l] : NULL};
    rc = layer_bwd_impl(n, rowptr, colidx, val, dims[l], dims[l + 1], ord, own_relu,
                        l == 0 ? X : H[l], l == 0 ? ldx : dims[l], H[l + 1], dims[l + 1], G,
                        dims[l + 1], W[l], dims[l + 1], W_G[l], dims[l + 1], HG, dims[l], &qf, &qb);
    free(G);
    G = HG;
  }
  free(G);
  for (int l = 1; l <= L; ++l) free(H[l]);
  free(H);
  return rc;
}

int mggcn_ref_epoch(int n, const int32_t* rowptr, const int32_t* colidx, const double* val, int L,
                    const int32_t* dims, const int32_t* orders, const double* X, int64_t ldx,
                    const int32_t* labels, const double* const* W, double* loss, double* const* W_G,
                    double* logits_out, const uint8_t* const* relu_masks) {
  return epoch_impl(n, rowptr, colidx, val, L, dims, orders, X, ldx, labels, W, loss, W_G, logits_out,
                    relu_masks, 0, NULL, NULL, NULL, NULL);
}

/* The same epoch with every SpMM gathering a bfloat16 copy of its dense operand (see RefGather).
 * Per layer l the operand of the forward SpMM is n x (dims[l+1] if GeMM first, dims[l] if SpMM
 * first), that of the backward SpMM n x (dims[l+1] if GeMM first: the gradient Z_G; dims[l] if
 * SpMM first: U = Z_G W^T, formed only for l > 0).  fwd_in / bwd_in: NULL, or L pointers (each
 * NULL or dense codes, ld = width) to use as those operands; fwd_out / bwd_out: NULL, or L
 * pointers (each NULL or room for the codes) that receive the oracle's own roundings.
 * Gradients treat the rounding as the identity (it is applied to values, not differentiated).
 */
int mggcn_ref_epoch_bf16(int n, const int32_t* rowptr, const int32_t* colidx, const double* val, int L,
                         const int32_t* dims, const int32_t* orders, const double* X, int64_t ldx,
                         const int32_t* labels, const double* const* W, double* loss, double* const* W_G,
                         double* logits_out, const uint8_t* const* relu_masks,
                         const uint16_t* const* fwd_in, const uint16_t* const* bwd_in,
                         uint16_t* const* fwd_out, uint16_t* const* bwd_out) {
  return epoch_impl(n, rowptr, colidx, val, L, dims, orders, X, ldx, labels, W, loss, W_G, logits_out,
                    relu_masks, 1, fwd_in, bwd_in, fwd_out, bwd_out);
}

/* ------------------------------------------------------------------------
 * Adam update (the optimiser the paper trains with; it states no hyper-parameters, so they are
 * arguments).  Textbook form with bias correction, t = 1, 2, ...:
 *   m <- b1 m + (1-b1) g ;  v <- b2 v + (1-b2) g^2
 *   W <- W - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
 * --------------------------------------------------------------------- */
int mggcn_ref_adam_step(int64_t count, double* W, const double* G, double* m, double* v, int t, double lr,
                        double b1, double b2, double eps) {
  if (count < 0 || t < 1) return REF_E_ARG;
  const double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
  for (int64_t i = 0; i < count; ++i) {
    m[i] = b1 * m[i] + (1.0 - b1) * G[i];
    v[i] = b2 * v[i] + (1.0 - b2) * G[i] * G[i];
    W[i] -= lr * (m[i] / c1) / (sqrt(v[i] / c2) + eps);
  }
  return REF_OK;
}
